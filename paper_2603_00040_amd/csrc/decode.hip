// Alg. 1 for decode steps over the NVFP4 KV cache: a (sequence, kv head) has at most 16 query rows (the G query heads of
// its group times the few newest positions), so the step is bound by reading the cache once, and the work of a launch is
// as uneven as the sequences are long.  The keys of a sequence are therefore cut into chunks of CK keys that workgroups
// take from a queue, and three facts keep the result that of Alg. 1 in key-tile order:
//   * P-tilde of key tile j is exp(S - m_j) with m_j the running row maximum after tile j, and phi is applied to that.
//     m_j needs nothing but the scores: a chunk first computes its scores S = Q^F K^F^T (kept in LDS; only the K half of
//     its pages is read), publishes its row maxima, and takes the maxima of the chunks before it from memory.  With the
//     maximum m_0 at its first key known, every m_j inside the chunk follows, and the second half of the chunk's work
//     (softmax, phi(P-tilde), P^F V^F; the V half of its pages) runs exactly as it would after its predecessors.
//   * O and l are sums over key tiles of terms scaled by exp(m_j - m_final): partial sums may be formed per wave and per
//     chunk in units of their own last maximum and re-based when they are added (the rescaling of Alg. 1, regrouped).
//   * A chunk waits only for chunks of lower queue position (tickets are handed out in chunk-major order by an atomic
//     counter), and whoever holds a ticket is running: the holder of the lowest unfinished ticket never waits, so every
//     wait ends.  The wait is bounded all the same (spin_limit polls; on expiry an error word is set and the kernel
//     finishes with that chunk's maxima missing).
// K and V^F stream from the pages into registers (a lane takes 32 d of one key: 16 bytes of codes and two scale bytes) and
// are dequantized by the hardware conversions and a packed multiplication by the block scale.  S^T = K^F Q^F^T and O^T += V^F^T P^F^T are
// v_mfma_f32_16x16x32_f16 products (16 rows suffice); V^F passes through a small per-wave LDS tile so that the transposing
// LDS read can hand the matrix instruction keys-contiguous operands.
#include "common.hpp"
#include "kernels.hpp"

namespace aq {

namespace {

constexpr int kDecRows = 16;          // most query rows of a (sequence, kv head)
constexpr int kDecSFloats = 4096;     // LDS floats for a chunk's scores: R * CK <= this
constexpr int kDecMaxTiles = 16;      // 64-key tiles per chunk (CK <= 1024)

__device__ inline float ld_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Codes and scale bytes of (key, 32-d group g) of one part (K or V) of a page: D/8 bytes of codes, D/64 scale bytes.
template <int D>
struct RawKV { uint32_t w[D / 32]; uint32_t sc; };

template <int D>
__device__ inline RawKV<D> load_raw(const unsigned char* part, int slot, int g, bool ok) {
    RawKV<D> r;
    if (!ok) {
#pragma unroll
        for (int i = 0; i < D / 32; ++i) r.w[i] = 0u;
        r.sc = 0u;
        return r;
    }
    if constexpr (D == 128) {
        const uint4v c = *reinterpret_cast<const uint4v*>(part + (size_t)slot * 64 + 16 * g);
        r.w[0] = c[0]; r.w[1] = c[1]; r.w[2] = c[2]; r.w[3] = c[3];
        r.sc = *reinterpret_cast<const uint16_t*>(part + 128 * 64 + (size_t)slot * 8 + 2 * g);
    } else {
        const uint2v c = *reinterpret_cast<const uint2v*>(part + (size_t)slot * 32 + 8 * g);
        r.w[0] = c[0]; r.w[1] = c[1];
        r.sc = part[128 * 32 + (size_t)slot * 4 + g];
    }
    return r;
}

// The 8 values d = (D/4) g + 8 s .. + 7 of the lane's key as fp16 (exact: code times E4M3 scale; the conversion's own scale
// operand only takes powers of two, so the block scale is a packed fp16 multiplication).
template <int D>
__device__ inline half8 dequant8(const RawKV<D>& r, int s) {
    const float sv = (D == 128 && s >= 2) ? __builtin_amdgcn_cvt_scalef32_f32_fp8(r.sc, 1.0f, 1)
                                          : __builtin_amdgcn_cvt_scalef32_f32_fp8(r.sc, 1.0f, 0);
    const half2v sc2 = __builtin_bit_cast(half2v, pack_f16x2(sv, sv));
    const uint32_t w = r.w[s];
    uint4v v;
    v[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0) * sc2);
    v[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1) * sc2);
    v[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2) * sc2);
    v[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3) * sc2);
    return __builtin_bit_cast(half8, v);
}

__global__ void zero_ints_kernel(int* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// MFMA operand layouts (v_mfma_f32_16x16x32_f16): lane l = c + 16 g.  A: row c, contraction indices 8 g .. 8 g + 7;
// B: column c, the same contraction indices; result: column c, rows 4 g .. 4 g + 3.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void decode_kernel(
    const half_t* __restrict__ Qh,           // [B*Hkv][128][D] fp16: phi(Q), row r = (query head of the group) * Lq + position; rows >= R zero
    const unsigned char* __restrict__ cache, int num_pages, const int* __restrict__ page_table, int max_pages,
    const int* __restrict__ kv_lens, int B, int Hkv, int Lq, int R, int CK, int NC, int spin_limit,
    int* ctl /* [0] ticket counter, [1] error word */, int* done, int* flags,
    float* cmax, float* part_o, float* part_l, float* part_m,        // shared between workgroups: no __restrict__
    uint16_t* __restrict__ O, float* __restrict__ lse, float c /* log2(e)/sqrt(d) */)
{
    constexpr int NS = D / 32;                 // contraction steps of S
    constexpr int NDT = D / 16;                // 16-row blocks of O^T
    constexpr int RS = 2 * D + 32;             // bytes per key of the V tile (padded: the transposing reads walk four rows)
    constexpr size_t HB = (size_t)2 * 128 * (D / 2 + D / 16);     // bytes per kv head in a page
    constexpr size_t VOFF = (size_t)128 * (D / 2 + D / 16);       // the V part behind the K part

    __shared__ float sbuf[kDecSFloats];                            // scores of the chunk [R][CK]
    __shared__ __align__(16) unsigned char stage[4 * 32 * RS];     // per wave: V^F of 32 keys [key][d] fp16; later the merge buffer
    __shared__ float tmax[kDecRows][kDecMaxTiles + 1];             // row maximum of every tile
    __shared__ float run[kDecRows][kDecMaxTiles + 1];              // running maximum after every tile
    __shared__ float red[16][kDecRows];
    __shared__ float lsum_w[4][kDecRows];
    __shared__ int s_ticket, s_old;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cc = lane & 15, g = lane >> 4;
    const int row = cc < R ? cc : 0;                               // lanes of unused columns follow row 0 (never stored)
    const int nunits = NC * B * Hkv;
    float* mbuf = reinterpret_cast<float*>(stage);                 // [4][R][D] when the waves' partial sums are added

    for (;;) {
        __syncthreads();
        if (tid == 0) s_ticket = atomicAdd(&ctl[0], 1);
        __syncthreads();
        const int ticket = s_ticket;
        if (ticket >= nunits) break;
        const int ch = ticket / (B * Hkv), bh = ticket % (B * Hkv), b = bh / Hkv, h = bh % Hkv;
        const int Lk = min(kv_lens[b], max_pages * 128);
        if (Lk < 1) {                                              // no keys: O = 0, L = -inf
            if (ch == 0) {
                for (int e = tid; e < R * D; e += 256) O[(size_t)bh * R * D + e] = 0;
                if (tid < R) lse[(size_t)bh * R + tid] = -INFINITY;
            }
            continue;
        }
        const int nch = (Lk + CK - 1) / CK;
        if (ch >= nch) continue;
        const int key0 = ch * CK;
        const int NT = (min(CK, Lk - key0) + 63) / 64;
        const int klim = CAUSAL ? Lk - Lq + (row % Lq) : Lk - 1;   // last key this lane's row sees
        const int* table = page_table + (size_t)b * max_pages;

        // Q^F operand: row cc, d = (D/4) g + 8 s .. + 7
        half8 qreg[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qreg[s] = *reinterpret_cast<const half8*>(Qh + ((size_t)bh * 128 + cc) * D + (D / 4) * g + 8 * s);

        // The K (part_off = 0) or V part of tile t of the chunk, 16 keys per block: issued one tile ahead of its use.  Tiles
        // beyond the chunk, pages outside the cache and (V only) keys at or beyond the sequence's end read as zeros.
        auto fetch = [&](int t, size_t part_off, bool to_len, RawKV<D> (&raw)[4]) __attribute__((always_inline)) {
            const int k_t = key0 + 64 * t;
            const int page = t < NT ? table[k_t >> 7] : -1;
            const bool ok = page >= 0 && page < num_pages;
            const unsigned char* pp = cache + ((size_t)(ok ? page : 0) * Hkv + h) * HB + part_off;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
                raw[blk] = load_raw<D>(pp, (k_t & 127) + 16 * blk + cc, g, ok && (!to_len || k_t + 16 * blk + cc < Lk));
        };

        // ---- first half: scores of this wave's tiles into LDS, and their row maxima
        RawKV<D> nxt[4];
        fetch(wave, 0, false, nxt);
        for (int t = wave; t < NT; t += 4) {
            const int k_t = key0 + 64 * t;
            RawKV<D> raw[4];
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) raw[blk] = nxt[blk];
            fetch(t + 4, 0, false, nxt);
            float mx = -INFINITY;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int s = 0; s < NS; ++s)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(dequant8<D>(raw[blk], s), qreg[s], acc, 0, 0, 0);
                // acc[i]: key k_t + 16 blk + 4 g + i, row cc.  Masked keys (beyond the sequence, or after the query) get -inf
                // whatever the stale bytes of the page gave.
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (k_t + 16 * blk + 4 * g + i > klim) acc[i] = -INFINITY;
                    mx = fmaxf(mx, acc[i]);
                }
                if (cc < R) *reinterpret_cast<floatx4*>(&sbuf[cc * CK + 64 * t + 16 * blk + 4 * g]) = acc;
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            if (g == 0 && cc < R) tmax[cc][t] = mx;
        }
        fetch(wave, VOFF, true, nxt);            // the first V tile travels while the maxima are exchanged
        __syncthreads();

        // ---- the chunk's row maxima out, those of the chunks before it in
        const size_t unit = (size_t)bh * NC + ch;
        if (nch > 1) {
            if (tid < R) {
                float m = -INFINITY;
                for (int t = 0; t < NT; ++t) m = fmaxf(m, tmax[tid][t]);
                cmax[unit * kDecRows + tid] = m;
                __threadfence();
            }
            __syncthreads();
            if (tid == 0) __hip_atomic_store(&flags[unit], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        {
            const int r = tid & 15, i0 = tid >> 4;
            float m = -INFINITY;
            for (int i = i0; i < ch; i += 16) {
                const size_t pu = (size_t)bh * NC + i;
                int spins = 0;
                bool there = true;
                while (__hip_atomic_load(&flags[pu], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == 0) {
                    if (++spins > spin_limit) { there = false; break; }
                    __builtin_amdgcn_s_sleep(8);
                }
                if (there) m = fmaxf(m, ld_agent(&cmax[pu * kDecRows + r]));
                else __hip_atomic_store(&ctl[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            red[i0][r] = m;
        }
        __syncthreads();
        if (tid < R) {
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, red[i][tid]);
            for (int t = 0; t < NT; ++t) { m = fmaxf(m, tmax[tid][t]); run[tid][t] = m; }
        }
        __syncthreads();

        // ---- second half: this wave's tiles in increasing order; O and l in units of the wave's latest maximum
        floatx4 o[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[dt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        float lacc = 0.0f, m_prev = -INFINITY;
        unsigned char* stg = stage + wave * (32 * RS);
        const uint32_t tr_base = lds_addr_of(stg) + (uint32_t)((8 * g + (cc >> 2)) * RS + 8 * (cc & 3));
        for (int t = wave; t < NT; t += 4) {
            RawKV<D> raw[4];         // (keys at or beyond the sequence's end are zeros: their P is 0, but stale bytes may be NaN)
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) raw[blk] = nxt[blk];
            fetch(t + 4, VOFF, true, nxt);
            const float m = run[row][t];
            const float alpha = __builtin_amdgcn_exp2f((m_prev - m) * c);     // first tile: exp2(-inf) = 0 on sums that are 0
            const float ms = m * c;
            m_prev = m;
            lacc *= alpha;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) o[dt] *= alpha;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                // V^F of keys 32 hh .. + 31 of the tile into the wave's tile: lane (key cc of 16, group g) holds 32 d of its key
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    unsigned char* dst = stg + (16 * sub + cc) * RS + (D / 2) * g;
#pragma unroll
                    for (int s = 0; s < NS; ++s)
                        *reinterpret_cast<half8*>(dst + 16 * s) = dequant8<D>(raw[2 * hh + sub], s);
                }
                // P-tilde of keys 32 hh + 8 g .. + 7 for row cc, then phi^-1(phi(.)) in blocks of 16 keys (this lane and lane ^ 16)
                const float* sp = &sbuf[row * CK + 64 * t + 32 * hh + 8 * g];
                const floatx4 s0 = *reinterpret_cast<const floatx4*>(sp), s1 = *reinterpret_cast<const floatx4*>(sp + 4);
                float p[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(fmaf(s0[i], c, -ms));
                    p[4 + i] = __builtin_amdgcn_exp2f(fmaf(s1[i], c, -ms));
                }
                lacc += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                float amax = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
                amax = fmaxf(amax, __shfl_xor(amax, 16));
                // RNE_E4M3(amax / 6) by the hardware conversion and back (P-tilde <= 1: no saturation)
                typedef short short2v __attribute__((ext_vector_type(2)));
                short2v pk = {0, 0};
                pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, amax * (1.0f / 6.0f), amax * (1.0f / 6.0f), 1.0f, false);
                const float bsc = __builtin_amdgcn_cvt_scalef32_f32_fp8(__builtin_bit_cast(uint32_t, pk), 1.0f, 0);
                const float inv = fminf(__builtin_amdgcn_rcpf(bsc), 512.0f);      // a scale of 0: P^F is 0 whatever the codes
                float rq[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) rq[i] = p[i] * inv;
                uint32_t pf[4];
                fq_oct_f16(rq, pack_f16x2(bsc, bsc), pf);
                uint4v pfv; pfv[0] = pf[0]; pfv[1] = pf[1]; pfv[2] = pf[2]; pfv[3] = pf[3];
                const half8 bp = __builtin_bit_cast(half8, pfv);
                __builtin_amdgcn_wave_barrier();
                // O^T[d][row] += V^F^T[d][keys] P^F^T[keys][row]
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const uint2v lo = lds_read_tr16_at(tr_base + 32 * dt), hi = lds_read_tr16_at(tr_base + 32 * dt + 4 * RS);
                    uint4v av; av[0] = lo[0]; av[1] = lo[1]; av[2] = hi[0]; av[3] = hi[1];
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, av), bp, o[dt], 0, 0, 0);
                }
            }
        }
        lacc += __shfl_xor(lacc, 16);
        lacc += __shfl_xor(lacc, 32);

        // ---- the four waves' sums, re-based to the chunk's last maximum, are added in LDS
        const float m_end = run[row][NT - 1];
        const float f = __builtin_amdgcn_exp2f((m_prev - m_end) * c);      // a wave without tiles: exp2(-inf) = 0
        __syncthreads();                                                   // every wave is done with its V tile
        if (cc < R) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) mbuf[(wave * R + cc) * D + 16 * dt + 4 * g + i] = o[dt][i] * f;
            if (g == 0) lsum_w[wave][cc] = lacc * f;
        }
        __syncthreads();
        const float ln2c = c * 0.6931471805599453f;
        if (nch == 1) {
            for (int e = tid; e < R * D; e += 256) {
                const int r = e / D;
                const float l = (lsum_w[0][r] + lsum_w[1][r]) + (lsum_w[2][r] + lsum_w[3][r]);
                const float v = (mbuf[e] + mbuf[R * D + e]) + (mbuf[2 * R * D + e] + mbuf[3 * R * D + e]);
                O[(size_t)bh * R * D + e] = f32_to_bf16_rne(v / l);
            }
            if (tid < R) {
                const float l = (lsum_w[0][tid] + lsum_w[1][tid]) + (lsum_w[2][tid] + lsum_w[3][tid]);
                lse[(size_t)bh * R + tid] = run[tid][NT - 1] * ln2c + logf(l);
            }
            continue;
        }
        for (int e = tid; e < R * D; e += 256)
            part_o[unit * kDecRows * D + e] = (mbuf[e] + mbuf[R * D + e]) + (mbuf[2 * R * D + e] + mbuf[3 * R * D + e]);
        if (tid < R) {
            part_l[unit * kDecRows + tid] = (lsum_w[0][tid] + lsum_w[1][tid]) + (lsum_w[2][tid] + lsum_w[3][tid]);
            part_m[unit * kDecRows + tid] = run[tid][NT - 1];
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) s_old = __hip_atomic_fetch_add(&done[bh], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (s_old != nch - 1) continue;
        // ---- the chunk that finishes last adds the chunks of its (sequence, kv head)
        __threadfence();
        for (int e = tid; e < R * D; e += 256) {
            const int r = e / D;
            const size_t u0 = (size_t)bh * NC;
            float M = -INFINITY;
            for (int i = 0; i < nch; ++i) M = fmaxf(M, ld_agent(&part_m[(u0 + i) * kDecRows + r]));
            float v = 0.0f, l = 0.0f;
            for (int i = 0; i < nch; ++i) {
                const float w = __builtin_amdgcn_exp2f((ld_agent(&part_m[(u0 + i) * kDecRows + r]) - M) * c);
                v += ld_agent(&part_o[(u0 + i) * kDecRows * D + e]) * w;
                l += ld_agent(&part_l[(u0 + i) * kDecRows + r]) * w;
            }
            O[(size_t)bh * R * D + e] = f32_to_bf16_rne(v / l);
            if (e % D == 0) lse[(size_t)bh * R + r] = M * ln2c + logf(l);
        }
    }
}

}  // namespace

// Keys per chunk for R rows per (sequence, kv head): the chunk's scores [R][CK] fp32 fit the LDS set aside for them.
int decode_chunk_keys(int R) { return max(256, min(1024, (kDecSFloats / R) / 128 * 128)); }
int decode_max_rows() { return kDecRows; }

size_t decode_ws_bytes(int B, int Hkv, int R, int max_pages, int D)
{
    const size_t CK = decode_chunk_keys(R), NC = ((size_t)max_pages * 128 + CK - 1) / CK, units = (size_t)B * Hkv * NC;
    size_t n = 256;                                                   // ticket counter and error word
    n += (((size_t)B * Hkv + units) * 4 + 255) / 256 * 256;            // chunks done per (sequence, kv head); a flag per chunk
    n += units * kDecRows * 4 * 3;                                     // row maxima; l and m of the partial sums
    n += units * kDecRows * D * 4;                                     // O of the partial sums
    return n;
}

int launch_decode(const void* qh, const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                  int B, int Hq, int Hkv, int Lq, int D, bool causal, void* ws, int spin_limit, void* o, float* lse, hipStream_t st)
{
    const int R = (Hq / Hkv) * Lq;
    if (R < 1 || R > kDecRows || (D != 64 && D != 128)) return -1;
    const int CK = decode_chunk_keys(R), NC = (max_pages * 128 + CK - 1) / CK;
    const size_t units = (size_t)B * Hkv * NC;
    if (units > 0x7FFFFFFFull) return -1;
    unsigned char* p = (unsigned char*)ws;
    int* ctl = (int*)p;                      p += 256;
    int* done = (int*)p;
    int* flags = done + (size_t)B * Hkv;     p += (((size_t)B * Hkv + units) * 4 + 255) / 256 * 256;
    float* cmax = (float*)p;                 p += units * kDecRows * 4;
    float* part_l = (float*)p;               p += units * kDecRows * 4;
    float* part_m = (float*)p;               p += units * kDecRows * 4;
    float* part_o = (float*)p;
    const int nz = 64 + (int)((size_t)B * Hkv + units);       // the control words are one run of ints from ctl on
    hipLaunchKernelGGL(zero_ints_kernel, dim3((nz + 255) / 256), dim3(256), 0, st, ctl, nz);
    if (hipGetLastError() != hipSuccess) return -1;
    static int ncu[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    int cus = __atomic_load_n(&ncu[dev & 63], __ATOMIC_RELAXED);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        __atomic_store_n(&ncu[dev & 63], cus, __ATOMIC_RELAXED);
    }
    const unsigned grid = (unsigned)min((size_t)2 * cus, units);
    const float c = 1.4426950408889634f / sqrtf((float)D);
#define AQ_DEC(DD, C) hipLaunchKernelGGL((decode_kernel<DD, C>), dim3(grid), dim3(256), 0, st, (const half_t*)qh, (const unsigned char*)cache, \
        num_pages, page_table, max_pages, kv_lens, B, Hkv, Lq, R, CK, NC, spin_limit, ctl, done, flags, cmax, part_o, part_l, part_m, \
        (uint16_t*)o, lse, c)
    if (D == 128) { if (causal) AQ_DEC(128, true); else AQ_DEC(128, false); }
    else          { if (causal) AQ_DEC(64, true); else AQ_DEC(64, false); }
#undef AQ_DEC
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace aq
