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
//     chunk in units of their own last maximum and re-based when they are added (the rescaling of Alg. 1, regrouped): the
//     waves' in LDS, the chunks' by a small second kernel.
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

// The row maxima that chunks hand to each other travel as relaxed device-scope 64-bit atomic stores and loads, value and
// "present" tag in one word: such accesses are performed where all XCDs see them (the L2 of an XCD is not coherent with the
// others for ordinary accesses) and need no release or acquire fence at device scope.  Such a fence writes back the whole
// L2, and with every workgroup issuing a few per chunk it was most of the kernel's time (0.86 ms for a step of 0.1 ms).

// Codes and scale bytes of (key, 32-d group g) of one part (K or V) of a page: D/8 bytes of codes, D/64 scale bytes.
template <int D>
struct RawKV { uint32_t w[D / 32]; uint32_t sc; };

template <int D>
__device__ inline RawKV<D> load_raw(const unsigned char* part, int slot, int g) {
    RawKV<D> r;
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

// The block scales of a lane's 32 d (two E4M3 bytes; one for D = 64) as an fp16 pair, by one conversion.
// `live` false: the key does not exist (beyond the sequence, or a page outside the cache): scales of 0 make its values 0
// whatever was read (the codes are finite by construction, the scale bytes need not be).
template <int D>
__device__ inline half2v scales_of(const RawKV<D>& r, bool live) {
    return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(live ? r.sc : 0u, 1.0f, false);
}

// The 8 values d = (D/4) g + 8 s .. + 7 of the lane's key as fp16 (exact: code times E4M3 scale; the conversion's own scale
// operand only takes powers of two, so the block scale is a packed fp16 multiplication).
template <int D>
__device__ inline half8 dequant8(const RawKV<D>& r, half2v sc, int s) {
    const half_t sv = (D == 128 && s >= 2) ? sc[1] : sc[0];
    const half2v sc2 = {sv, sv};
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
__global__ __launch_bounds__(256, 2) void decode_kernel(
    const half_t* __restrict__ Qh,           // [B*Hkv][128][D] fp16: phi(Q), row r = (query head of the group) * Lq + position; rows >= R zero
    const unsigned char* __restrict__ cache, int num_pages, const int* __restrict__ page_table, int max_pages,
    const int* __restrict__ kv_lens, int B, int Hkv, int Lq, int R, int CK, int NC, int spin_limit,
    int* ctl /* [0] ticket counter, [1] error word */,
    unsigned long long* cmax /* per chunk and row: {1, row maximum} once known, 0 before */,
    float* part_o, float* part_l, float* part_m,        // shared between workgroups: no __restrict__
    uint16_t* __restrict__ O, float* __restrict__ lse, float c /* log2(e)/sqrt(d) */)
{
    constexpr int NS = D / 32;                 // contraction steps of S
    constexpr int NDT = D / 16;                // 16-row blocks of O^T
    constexpr int RS = 2 * D + 16;             // bytes per key of the V tile (padded: 16 rows are written side by side)
    constexpr int PS = 144;                    // bytes per row of the P^F tile (64 keys, padded: 16 rows are read side by side)
    constexpr size_t HB = (size_t)2 * 128 * (D / 2 + D / 16);     // bytes per kv head in a page
    constexpr size_t VOFF = (size_t)128 * (D / 2 + D / 16);       // the V part behind the K part

    __shared__ float sbuf[kDecSFloats];                            // scores of the chunk [R][CK]
    __shared__ __align__(16) unsigned char stage[4 * 32 * RS];     // per wave: V^F of 32 keys [key][d] fp16; later the merge buffer
    __shared__ __align__(16) unsigned char pfb[4 * kDecRows * PS]; // per wave: P^F of a tile [row][key] fp16
    __shared__ float tmax[kDecRows][kDecMaxTiles + 1];             // row maximum of every tile
    __shared__ float run[kDecRows][kDecMaxTiles + 1];              // running maximum after every tile
    __shared__ float red[16][kDecRows];
    __shared__ float lsum_w[4][kDecRows];
    __shared__ int s_ticket;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cc = lane & 15, g = lane >> 4;
    const int row = cc < R ? cc : 0;                               // lanes of unused columns follow row 0 (never stored)
    const int nunits = NC * B * Hkv;
    float* mbuf = reinterpret_cast<float*>(stage);                 // [4][R][D] when the waves' partial sums are added

    // A trip to memory and back takes microseconds, a chunk's own work about ten: what a chunk needs from memory is asked for
    // as early as its address is known (the next ticket while this chunk is in work, the maxima of the chunks in front before
    // this chunk's scores, the first V tiles before the exchange of maxima).
    int next_ticket = 0;
    if (tid == 0) next_ticket = atomicAdd(&ctl[0], 1);
    for (;;) {
        __syncthreads();
        if (tid == 0) s_ticket = next_ticket;
        __syncthreads();
        const int ticket = s_ticket;
        if (ticket >= nunits) break;
        if (tid == 0) next_ticket = atomicAdd(&ctl[0], 1);
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
        const int klim_min = CAUSAL ? Lk - Lq : Lk - 1;            // ... and the least of those over the rows
        const int* table = page_table + (size_t)b * max_pages;

        // the row maxima of the chunks in front, as far as they are there already (they almost always are)
        const int pr = tid & 15, pi0 = tid >> 4;
        float m_pred = -INFINITY;
        bool pred_missing = false;
        if (pr < R) {
            for (int i = pi0; i < ch; i += 16) {
                const unsigned long long v = __hip_atomic_load(&cmax[((size_t)bh * NC + i) * kDecRows + pr], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v >> 32) m_pred = fmaxf(m_pred, __uint_as_float((uint32_t)v));
                else pred_missing = true;
            }
        }

        // Q^F operand: row cc, d = (D/4) g + 8 s .. + 7
        half8 qreg[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qreg[s] = *reinterpret_cast<const half8*>(Qh + ((size_t)bh * 128 + cc) * D + (D / 4) * g + 8 * s);

        // This wave's tiles of the chunk are tiles wave, wave + 4, wave + 8, wave + 12 (at most 4: CK <= 1024), and what it
        // reads is the sequence K part of tile 0, 1, 2, 3, then V part of tile 0, 1, 2, 3.  Three items of that sequence are
        // always in flight (13.5 KiB per wave; a step of this kind lives on the bytes it keeps in flight): item i + 3 is
        // requested when item i has been consumed, into the registers that held it.  The loads are unconditional and sit in
        // straight-line code with the tile loops unrolled (a tile that does not exist reads the chunk's last tile again, a
        // page id outside the cache reads page 0; what they return is discarded or zeroed at its use): only then can the
        // compiler count them and wait for exactly the item it is about to use.  (With the requests under branches, or with
        // the buffers rotated by register copies, it waited for everything in flight at every tile.)
        const unsigned char* tile_src[4];
        bool tile_ok[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int k_t = key0 + 64 * min(wave + 4 * it, NT - 1);
            const int page = table[k_t >> 7];
            tile_ok[it] = page >= 0 && page < num_pages;
            tile_src[it] = cache + ((size_t)(tile_ok[it] ? page : 0) * Hkv + h) * HB;
        }
        RawKV<D> rw[3][4];
        auto issue = [&](int item) __attribute__((always_inline)) {         // item: a compile-time constant after unrolling
            const int it = item & 3;
            const int k_t = key0 + 64 * min(wave + 4 * it, NT - 1);
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
                rw[item % 3][blk] = load_raw<D>(tile_src[it] + (item >= 4 ? VOFF : 0), (k_t & 127) + 16 * blk + cc, g);
        };
        issue(0); issue(1); issue(2);

        // ---- first half: scores of this wave's tiles into LDS, and their row maxima
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int t = wave + 4 * it;
            if (t < NT) {
                const int k_t = key0 + 64 * t;
                float mx = -INFINITY;
                const bool need_mask = k_t + 63 > klim_min;                      // wave-uniform: only the chunk's last tile(s)
#pragma unroll
                for (int blk = 0; blk < 4; ++blk) {
                    floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
                    const half2v sc = scales_of<D>(rw[it % 3][blk], tile_ok[it]);
#pragma unroll
                    for (int s = 0; s < NS; ++s)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(dequant8<D>(rw[it % 3][blk], sc, s), qreg[s], acc, 0, 0, 0);
                    // acc[i]: key k_t + 16 blk + 4 g + i, row cc.  Masked keys (beyond the sequence, or after the query) get
                    // -inf whatever the stale bytes of the page gave.
                    if (need_mask) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (k_t + 16 * blk + 4 * g + i > klim) acc[i] = -INFINITY;
                    }
                    mx = max_nc(max_nc(mx, max_nc(acc[0], acc[1])), max_nc(acc[2], acc[3]));
                    if (cc < R) *reinterpret_cast<floatx4*>(&sbuf[cc * CK + 64 * t + 16 * blk + 4 * g]) = acc;
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                if (g == 0 && cc < R) tmax[cc][t] = mx;
            }
            issue(it + 3);                       // (the first V parts travel while the maxima are exchanged)
        }
        __syncthreads();

        // ---- the chunk's row maxima out, those of the chunks before it in
        const size_t unit = (size_t)bh * NC + ch;
        if (nch > 1 && tid < R) {
            float m = -INFINITY;
            for (int t = 0; t < NT; ++t) m = fmaxf(m, tmax[tid][t]);
            __hip_atomic_store(&cmax[unit * kDecRows + tid], (1ull << 32) | (unsigned long long)__float_as_uint(m),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (pred_missing) {              // wait for the ones that were not (bounded; see the head of this file)
            for (int i = pi0; i < ch; i += 16) {
                const unsigned long long* src = &cmax[((size_t)bh * NC + i) * kDecRows + pr];
                unsigned long long v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int spins = 0; (v >> 32) == 0 && spins < spin_limit; ++spins) {
                    __builtin_amdgcn_s_sleep(8);
                    v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (v >> 32) m_pred = fmaxf(m_pred, __uint_as_float((uint32_t)v));
                else __hip_atomic_store(&ctl[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        red[pi0][pr] = m_pred;
        __syncthreads();
        if (tid < R) {
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, red[i][tid]);
            for (int t = 0; t < NT; ++t) { m = fmaxf(m, tmax[tid][t]); run[tid][t] = m; }
        }
        __syncthreads();

        // ---- second half: this wave's tiles in increasing order; O and l in units of the wave's latest maximum.
        // Two lane maps.  The products want lane (cc, g) = query row cc, keys 8 g .. 8 g + 7 of half a tile, which for R rows
        // leaves 16 - R of 16 lanes idle; the softmax and phi(P-tilde), most of the vector work, therefore run in passes over
        // four rows with lane (q, j) = row 4 pass + q, keys 4 j .. 4 j + 3 of the tile (a block of 16 keys = 4 neighbouring
        // lanes), and hand P^F to the products through a small tile in LDS.
        floatx4 o[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[dt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        float m_prev = -INFINITY;
        float lacc[4] = {0.0f, 0.0f, 0.0f, 0.0f}, mp_prev[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        unsigned char* stg = stage + wave * (32 * RS);
        const uint32_t tr_base = lds_addr_of(stg) + (uint32_t)((8 * g + (cc >> 2)) * RS + 8 * (cc & 3));
        unsigned char* pfw = pfb + wave * (kDecRows * PS);
        const int pq = lane >> 4, pj = lane & 15;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int t = wave + 4 * it;
            if (t >= NT) break;
            const int k_t = key0 + 64 * t;
            RawKV<D> (&raw)[4] = rw[(it + 4) % 3];
            // P^F of the whole tile, four rows at a time
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                if (4 * ps < R) {
                    const int prow = min(4 * ps + pq, R - 1);
                    const float mrow = run[prow][t], ms = mrow * c;
                    const floatx4 sv = *reinterpret_cast<const floatx4*>(&sbuf[prow * CK + 64 * t + 4 * pj]);
                    float pt[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) pt[i] = __builtin_amdgcn_exp2f(fmaf(sv[i], c, -ms));
                    lacc[ps] = fmaf(lacc[ps], __builtin_amdgcn_exp2f((mp_prev[ps] - mrow) * c), (pt[0] + pt[1]) + (pt[2] + pt[3]));
                    mp_prev[ps] = mrow;
                    float amax = fmaxf(fmaxf(pt[0], pt[1]), fmaxf(pt[2], pt[3]));
                    amax = fmaxf(amax, __shfl_xor(amax, 1));
                    amax = fmaxf(amax, __shfl_xor(amax, 2));
                    // RNE_E4M3(amax / 6) by the hardware conversion and back (P-tilde <= 1: no saturation)
                    typedef short short2v __attribute__((ext_vector_type(2)));
                    short2v pk = {0, 0};
                    pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, amax * (1.0f / 6.0f), amax * (1.0f / 6.0f), 1.0f, false);
                    const uint32_t pkw = __builtin_bit_cast(uint32_t, pk);
                    const float bsc = __builtin_amdgcn_cvt_scalef32_f32_fp8(pkw, 1.0f, 0);
                    const half2v sc2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(pkw, 1.0f, false);      // (bsc, bsc)
                    const float inv = fminf(__builtin_amdgcn_rcpf(bsc), 512.0f);      // a scale of 0: P^F is 0 whatever the codes
                    uint32_t codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pkw, pt[0] * inv, pt[1] * inv, 1.0f, 0);
                    codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, pt[2] * inv, pt[3] * inv, 1.0f, 1);
                    uint2v w;
                    w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 0) * sc2);
                    w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 1) * sc2);
                    *reinterpret_cast<uint2v*>(pfw + (4 * ps + pq) * PS + 8 * pj) = w;
                }
            }
            const float m = run[row][t];
            const float alpha = __builtin_amdgcn_exp2f((m_prev - m) * c);     // first tile: exp2(-inf) = 0 on sums that are 0
            m_prev = m;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {            // rare after the chunk's first tiles
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) o[dt] *= alpha;
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                // V^F of keys 32 hh .. + 31 of the tile into the wave's tile: lane (key cc of 16, group g) holds 32 d of its key
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    unsigned char* dst = stg + (16 * sub + cc) * RS + (D / 2) * g;
                    // (keys at or beyond the sequence's end are zeros: their P is 0, but stale bytes may be NaN)
                    const half2v sc = scales_of<D>(raw[2 * hh + sub], tile_ok[it] && k_t + 32 * hh + 16 * sub + cc < Lk);
#pragma unroll
                    for (int s = 0; s < NS; ++s)
                        *reinterpret_cast<half8*>(dst + 16 * s) = dequant8<D>(raw[2 * hh + sub], sc, s);
                }
                __builtin_amdgcn_wave_barrier();
                // O^T[d][row] += V^F^T[d][keys] P^F^T[keys][row], keys 32 hh + 8 g .. + 7 in this lane
                const half8 bp = *reinterpret_cast<const half8*>(pfw + cc * PS + 64 * hh + 16 * g);
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const uint2v lo = lds_read_tr16_at(tr_base + 32 * dt), hi = lds_read_tr16_at(tr_base + 32 * dt + 4 * RS);
                    uint4v av; av[0] = lo[0]; av[1] = lo[1]; av[2] = hi[0]; av[3] = hi[1];
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, av), bp, o[dt], 0, 0, 0);
                }
            }
            if (it == 0) issue(7);
        }

        // ---- the four waves' sums, re-based to the chunk's last maximum, are added in LDS
        const float m_end = run[row][NT - 1];
        const float f = __builtin_amdgcn_exp2f((m_prev - m_end) * c);      // a wave without tiles: exp2(-inf) = 0
        __syncthreads();                                                   // every wave is done with its V tile
        if (cc < R) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) mbuf[(wave * R + cc) * D + 16 * dt + 4 * g + i] = o[dt][i] * f;
        }
#pragma unroll
        for (int ps = 0; ps < 4; ++ps) {
            if (4 * ps < R) {
                const int prow = min(4 * ps + pq, R - 1);
                float l = lacc[ps] * __builtin_amdgcn_exp2f((mp_prev[ps] - run[prow][NT - 1]) * c);
                l += __shfl_xor(l, 1); l += __shfl_xor(l, 2); l += __shfl_xor(l, 4); l += __shfl_xor(l, 8);
                if (pj == 0 && 4 * ps + pq < R) lsum_w[wave][4 * ps + pq] = l;
            }
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
        // several chunks: the partial sums go to memory for the kernel that adds them
        for (int e = tid; e < R * D; e += 256)
            part_o[unit * kDecRows * D + e] = (mbuf[e] + mbuf[R * D + e]) + (mbuf[2 * R * D + e] + mbuf[3 * R * D + e]);
        if (tid < R) {
            part_l[unit * kDecRows + tid] = (lsum_w[0][tid] + lsum_w[1][tid]) + (lsum_w[2][tid] + lsum_w[3][tid]);
            part_m[unit * kDecRows + tid] = run[tid][NT - 1];
        }
    }
}

// O and L of the (sequence, kv head)s whose keys were cut into several chunks: the chunks' partial sums, re-based to the last
// maximum.  A kernel of its own: the end of the first one is what makes the partial sums visible.
template <int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(
    const int* __restrict__ kv_lens, int Hkv, int R, int CK, int NC, int max_pages,
    const float* __restrict__ part_o, const float* __restrict__ part_l, const float* __restrict__ part_m,
    uint16_t* __restrict__ O, float* __restrict__ lse, float c)
{
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int Lk = min(kv_lens[bh / Hkv], max_pages * 128);
    const int nch = (Lk + CK - 1) / CK;
    if (nch < 2) return;
    const size_t u0 = (size_t)bh * NC;
    // (eight chunks per round, their loads issued together: one trip to memory per round instead of one per chunk)
    for (int e = tid; e < R * D; e += 256) {
        const int r = e / D;
        float M = -INFINITY, v = 0.0f, l = 0.0f;
        for (int i0 = 0; i0 < nch; i0 += 8) {
            float pm[8], po[8], pl[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const size_t u = u0 + min(i0 + k, nch - 1);
                pm[k] = i0 + k < nch ? part_m[u * kDecRows + r] : -INFINITY;
                po[k] = part_o[u * kDecRows * D + e];
                pl[k] = part_l[u * kDecRows + r];
            }
            float Mn = M;
#pragma unroll
            for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, pm[k]);
            const float a = __builtin_amdgcn_exp2f((M - Mn) * c);      // first round: exp2(-inf) = 0 on sums that are 0
            v *= a; l *= a; M = Mn;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float w = __builtin_amdgcn_exp2f((pm[k] - M) * c);      // a chunk that does not exist: weight 0
                v = fmaf(po[k], w, v);
                l = fmaf(pl[k], w, l);
            }
        }
        O[(size_t)bh * R * D + e] = f32_to_bf16_rne(v / l);
        if (e % D == 0) lse[(size_t)bh * R + r] = M * (c * 0.6931471805599453f) + logf(l);
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
    n += units * kDecRows * 8;                                         // row maxima with their tags
    n += units * kDecRows * 4 * 2;                                     // l and m of the partial sums
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
    unsigned long long* cmax = (unsigned long long*)p;     p += units * kDecRows * 8;
    float* part_l = (float*)p;               p += units * kDecRows * 4;
    float* part_m = (float*)p;               p += units * kDecRows * 4;
    float* part_o = (float*)p;
    // the counters and the tagged row maxima are one run of ints from ctl on
    const size_t nz64 = ((unsigned char*)cmax - (unsigned char*)ctl) / 4 + units * kDecRows * 2;
    if (nz64 > 0x7FFFFFFFull) return -1;
    const int nz = (int)nz64;
    hipLaunchKernelGGL(zero_ints_kernel, dim3((nz + 255) / 256), dim3(256), 0, st, ctl, nz);
    if (hipGetLastError() != hipSuccess) return -1;
    const int cus = device_cu_count();
    const unsigned grid = (unsigned)min((size_t)2 * cus, units);
    const float c = 1.4426950408889634f / sqrtf((float)D);
#define AQ_DEC(DD, C) hipLaunchKernelGGL((decode_kernel<DD, C>), dim3(grid), dim3(256), 0, st, (const half_t*)qh, (const unsigned char*)cache, \
        num_pages, page_table, max_pages, kv_lens, B, Hkv, Lq, R, CK, NC, spin_limit, ctl, cmax, part_o, part_l, part_m, \
        (uint16_t*)o, lse, c)
    if (D == 128) { if (causal) AQ_DEC(128, true); else AQ_DEC(128, false); }
    else          { if (causal) AQ_DEC(64, true); else AQ_DEC(64, false); }
#undef AQ_DEC
    if (hipGetLastError() != hipSuccess) return -1;
    if (NC > 1) {
        if (D == 128) hipLaunchKernelGGL((decode_merge_kernel<128>), dim3(B * Hkv), dim3(256), 0, st, kv_lens, Hkv, R, CK, NC, max_pages,
                                         part_o, part_l, part_m, (uint16_t*)o, lse, c);
        else          hipLaunchKernelGGL((decode_merge_kernel<64>), dim3(B * Hkv), dim3(256), 0, st, kv_lens, Hkv, R, CK, NC, max_pages,
                                         part_o, part_l, part_m, (uint16_t*)o, lse, c);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace aq
