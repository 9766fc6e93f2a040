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
// The queue holds only chunks that exist: a small kernel in front lists them (sequence, kv head, chunk, key count) in
// chunk-major order, so that a ticket is one 16-byte read away from everything a workgroup needs to know, and a workgroup
// knows its next chunk while it works on the current one: the next chunk's first K tiles and its query rows are requested
// during the second half of the current chunk, and the stream from the cache never stops at a chunk boundary.
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
constexpr int kDecItemInts = 16;      // ints per entry of the list of chunks

// The row maxima that chunks hand to each other travel as relaxed device-scope 64-bit atomic stores and loads, value and
// "present" tag in one word: such accesses are performed where all XCDs see them (the L2 of an XCD is not coherent with the
// others for ordinary accesses) and need no release or acquire fence at device scope.  Such a fence writes back the whole
// L2, and with every workgroup issuing a few per chunk it was most of the kernel's time (0.86 ms for a step of 0.1 ms).

// Codes and scale bytes of (key, 32-d group g) of one part (K or V) of a page: D/8 bytes of codes, D/64 scale bytes.
template <int D>
struct RawKV { uint32_t w[D / 32]; uint32_t sc; };

// `part`: the K or V part of a page's head plus the tile's first key (wave-uniform); code_off / scale_off: this lane's byte
// offsets for key cc of the first 16 keys, group g (32-bit: a uniform base and a lane offset is an addressing mode of the
// load, a per-lane 64-bit address is two more vector instructions per load); blk: which 16 keys of the tile.
template <int D>
__device__ inline RawKV<D> load_raw(const unsigned char* part, uint32_t code_off, uint32_t scale_off, int blk) {
    RawKV<D> r;
    if constexpr (D == 128) {
        const uint4v c = *reinterpret_cast<const uint4v*>(part + (code_off + 16u * 64u * blk));
        r.w[0] = c[0]; r.w[1] = c[1]; r.w[2] = c[2]; r.w[3] = c[3];
        r.sc = *reinterpret_cast<const uint16_t*>(part + (scale_off + 16u * 8u * blk));
    } else {
        const uint2v c = *reinterpret_cast<const uint2v*>(part + (code_off + 16u * 32u * blk));
        r.w[0] = c[0]; r.w[1] = c[1];
        r.sc = part[scale_off + 16u * 4u * blk];
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

// Before every step: clears the queue's counters and the tagged row maxima (ints [0, nz) from ctl on, except ctl[2]), and
// workgroup 0 lists the chunks that exist, in chunk-major order, as items of kDecItemInts ints {sequence, kv head, chunk,
// keys of the sequence, the page ids of the chunk's (at most 8) pages, -1 where the sequence has none}, their number going
// to ctl[2].  A (sequence, kv head) without keys gets its result here: O = 0, L = -inf.
__global__ __launch_bounds__(256) void decode_plan_kernel(const int* __restrict__ kv_lens, const int* __restrict__ page_table,
                                                          int B, int Hkv, int R, int D, int CK, int NC,
                                                          int max_pages, int* __restrict__ ctl, int nz, int* __restrict__ work,
                                                          uint16_t* __restrict__ O, float* __restrict__ lse)
{
    const int tid = threadIdx.x;
    const int gi = blockIdx.x * 256 + tid;
    if (gi < nz && gi != 2) ctl[gi] = 0;
    if (blockIdx.x != 0) return;
    __shared__ int cnt[4];
    __shared__ int lens_s[2048];
    const int BH = B * Hkv;
    const bool staged = B <= 2048;                            // the sequences' key counts, next to the lanes that walk over them
    if (staged)
        for (int i = tid; i < B; i += 256) lens_s[i] = min(kv_lens[i], max_pages * 128);
    __syncthreads();
    const int P = NC * B;                                     // pair p = chunk * B + sequence; its Hkv heads are neighbours in the list
    const int per = (P + 255) / 256;                          // (the host has checked that NC * B * Hkv fits an int)
    const int p0 = min(P, tid * per), p1 = min(P, p0 + per);
    auto walk = [&](auto&& visit) __attribute__((always_inline)) {
        if (p0 >= p1) return;
        int ch = p0 / B, b = p0 % B;
        for (int q = p0; q < p1; ++q) {
            const int Lk = staged ? lens_s[b] : min(kv_lens[b], max_pages * 128);
            if (Lk >= 1 && (long long)ch * CK < Lk) visit(b, ch, Lk);
            if (++b == B) { b = 0; ++ch; }
        }
    };
    int n = 0;
    walk([&](int, int, int) { ++n; });
    // inclusive prefix sums: inside each wave by shuffles, then the four waves' totals
    int incl = n;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if ((tid & 63) >= d) incl += up;
    }
    if ((tid & 63) == 63) cnt[tid >> 6] = incl;
    __syncthreads();
    for (int w = 0; w < (tid >> 6); ++w) incl += cnt[w];
    const int total = cnt[0] + cnt[1] + cnt[2] + cnt[3];
    size_t pos = (size_t)(incl - n) * Hkv;
    walk([&](int b, int ch, int Lk) {
        int pg[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int pi = ch * (CK / 128) + j;
            pg[j] = pi < max_pages && pi * 128 < Lk ? page_table[(size_t)b * max_pages + pi] : -1;
        }
        for (int h = 0; h < Hkv; ++h) {
            int4* item = reinterpret_cast<int4*>(work + kDecItemInts * pos++);
            item[0] = make_int4(b, h, ch, Lk);
            item[1] = make_int4(pg[0], pg[1], pg[2], pg[3]);
            item[2] = make_int4(pg[4], pg[5], pg[6], pg[7]);
        }
    });
    if (tid == 0) ctl[2] = total * Hkv;
    for (int bh = tid; bh < BH; bh += 256) {
        if ((staged ? lens_s[bh / Hkv] : kv_lens[bh / Hkv]) < 1) {
            for (int e = 0; e < R * D; ++e) O[(size_t)bh * R * D + e] = 0;
            for (int r = 0; r < R; ++r) lse[(size_t)bh * R + r] = -INFINITY;
        }
    }
}

// MFMA operand layouts (v_mfma_f32_16x16x32_f16): lane l = c + 16 g.  A: row c, contraction indices 8 g .. 8 g + 7;
// B: column c, the same contraction indices; result: column c, rows 4 g .. 4 g + 3.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void decode_kernel(
    const half_t* __restrict__ Qh,           // [B*Hkv][128][D] fp16: phi(Q), row r = (query head of the group) * Lq + position; rows >= R zero
    const unsigned char* __restrict__ cache, int num_pages, int Hkv, int Lq, int R, int CK, int NC, int spin_limit,
    int* ctl /* [0] ticket counter, [1] error word, [2] number of chunks in the list */,
    const int* __restrict__ work /* the list of chunks, see decode_plan_kernel */,
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

    __shared__ __align__(16) float sbuf[kDecSFloats];              // scores of the chunk [R][CK]
    __shared__ __align__(16) unsigned char stage[4 * 32 * RS];     // per wave: V^F of 32 keys [key][d] fp16; later the merge buffer
    __shared__ __align__(16) unsigned char pfb[4 * kDecRows * PS]; // per wave: P^F of a tile [row][key] fp16
    __shared__ float tmax[kDecRows][kDecMaxTiles + 1];             // row maximum of every tile
    __shared__ float run[kDecRows][kDecMaxTiles + 1];              // running maximum after every tile
    __shared__ float lsum_w[4][kDecRows];
    __shared__ int s_ticket;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cc = lane & 15, g = lane >> 4;
    const int row = cc < R ? cc : 0;                               // lanes of unused columns follow row 0 (never stored)
    float* mbuf = reinterpret_cast<float*>(stage);                 // [4][R][D] when the waves' partial sums are added
    const uint32_t sbuf_ad = lds_addr_of(sbuf);
    const int nwork = __builtin_amdgcn_readfirstlane(ctl[2]);
    if (nwork < 1) return;

    // What a workgroup needs to know of a chunk (wave-uniform; the tiles are this wave's: tiles wave, wave + 4, wave + 8,
    // wave + 12 of the chunk, at most 4 since CK <= 1024).  A tile that does not exist stands for the chunk's last tile, a
    // page id outside the cache for page 0: what their loads return is discarded or zeroed at its use.  A ticket beyond the
    // list stands for the list's last chunk (its loads are dropped at the end of the kernel).
    struct Chunk {
        int b, h, ch, Lk, key0, NT;
        const unsigned char* src[4];       // head h of the tile's page
        int slot0[4];                      // first key of the tile within its page (chunks start at page boundaries)
        bool ok[4];
    };
    auto chunk_of = [&](int tk) __attribute__((always_inline)) -> Chunk {
        Chunk x;
        // (the whole item in one request: a page id picked by an address computed from the item would be a second trip)
        const int4* wi = reinterpret_cast<const int4*>(work + (size_t)kDecItemInts * min(tk, nwork - 1));
        const int4 w0 = wi[0], w1 = wi[1], w2 = wi[2];
        const int pg[8] = {w1.x, w1.y, w1.z, w1.w, w2.x, w2.y, w2.z, w2.w};
        x.b = w0.x; x.h = w0.y; x.ch = w0.z; x.Lk = w0.w;
        x.key0 = x.ch * CK;
        x.NT = (min(CK, x.Lk - x.key0) + 63) / 64;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int tt = min(wave + 4 * it, x.NT - 1), pi = tt >> 1;
            int page = pg[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) page = pi == j ? pg[j] : page;
            x.ok[it] = page >= 0 && page < num_pages;
            // (the tile's first key, 0 or 64 of its page, goes into the base: codes and scale bytes of a key are D/2 and D/16 bytes)
            x.src[it] = cache + ((size_t)(x.ok[it] ? page : 0) * Hkv + x.h) * HB;
            x.slot0[it] = 64 * (tt & 1);
        }
        return x;
    };

    // A trip to memory and back takes microseconds, a chunk's own work about ten: what a chunk needs from memory is asked for
    // as early as its address is known.  What a wave reads of a chunk is the sequence K part of its tile 0, 1, 2, 3, then V
    // part of tile 0, 1, 2, 3 (items 0 .. 7), and three items of that sequence, continued into the next chunk, are always in
    // flight (13.5 KiB per wave; a step of this kind lives on the bytes it keeps in flight): an item is requested into the
    // registers of an item that has just been consumed.  The loads are unconditional and sit in straight-line code with the
    // tile loops unrolled: only then can the compiler count them and wait for exactly the item it is about to use.  (With
    // the requests under branches, or with the buffers rotated by register copies, it waited for everything in flight at
    // every tile.)  Item i lives in slot i mod 3; the next chunk's items 2, 0, 1 are requested, in that order, as the slots
    // of this chunk's V parts fall free.
    RawKV<D> rw[3][4];
    const uint32_t code_off = (uint32_t)(cc * (D / 2) + (D / 8) * g);                       // key cc of a block of 16, 32-d group g
    const uint32_t scale_off = (uint32_t)(128 * (D / 2) + cc * (D / 16) + (D / 64) * g);
    auto issue = [&](const Chunk& x, int item) __attribute__((always_inline)) {     // item: a compile-time constant after unrolling
        const int it = item & 3;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            rw[item % 3][blk] = load_raw<D>(x.src[it] + (item >= 4 ? VOFF : 0), code_off + (uint32_t)x.slot0[it] * (D / 2),
                                            scale_off + (uint32_t)x.slot0[it] * (D / 16), blk);
    };
    // Q^F operand: row cc, d = (D/4) g + 8 s .. + 7
    half8 qreg[NS];
    auto load_q = [&](const Chunk& x) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qreg[s] = *reinterpret_cast<const half8*>(Qh + ((size_t)(x.b * Hkv + x.h) * 128 + cc) * D + (D / 4) * g + 8 * s);
    };

    int next_ticket = 0;
    if (tid == 0) s_ticket = atomicAdd(&ctl[0], 1);
    __syncthreads();
    int ticket = __builtin_amdgcn_readfirstlane(s_ticket);
    __syncthreads();
    if (tid == 0) next_ticket = atomicAdd(&ctl[0], 1);
    Chunk cur = chunk_of(ticket);
    load_q(cur);
    // (in this order, as at the end of the loop: the wait of the loop's first tile is the one both entries allow)
    __builtin_amdgcn_sched_barrier(0);
    issue(cur, 2);
    __builtin_amdgcn_sched_barrier(0);
    issue(cur, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue(cur, 1);
    __builtin_amdgcn_sched_barrier(0);

    while (ticket < nwork) {
        const int ch = cur.ch, bh = cur.b * Hkv + cur.h, Lk = cur.Lk, key0 = cur.key0, NT = cur.NT;
        const int nch = (Lk + CK - 1) / CK;
        const int klim = CAUSAL ? Lk - Lq + (row % Lq) : Lk - 1;   // last key this lane's row sees
        const int klim_min = CAUSAL ? Lk - Lq : Lk - 1;            // ... and the least of those over the rows

        // exchange map of the maxima: lane (xr, xt) = row xr, tile xt of this chunk / xt-th chunk in front (16 neighbouring lanes
        // per row: reductions and running maxima are shuffles)
        const int xr = tid >> 4, xt = tid & 15;
        unsigned long long v_early = 0;

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
                    const half2v sc = scales_of<D>(rw[it % 3][blk], cur.ok[it]);
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
                    // (CK is a multiple of 128: the address is a multiple of 16, which the compiler cannot see in an index)
                    if (cc < R) lds_write16_at(sbuf_ad + 4u * (uint32_t)(cc * CK + 64 * t + 16 * blk + 4 * g), __builtin_bit_cast(uint4v, acc));
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                if (g == 0 && cc < R) tmax[cc][t] = mx;
            }
            issue(cur, it + 3);                  // (the first V parts travel while the maxima are exchanged)
            // the row maximum of one chunk in front per lane, asked for in passing (unconditionally, like the items) and
            // looked at after the scores: by then it has arrived, and most of the time it is the maximum, not the empty slot
            if (it == 1)
                v_early = __hip_atomic_load(&cmax[((size_t)bh * NC + min(xt, max(ch - 1, 0))) * kDecRows + xr],
                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the next ticket (asked for a chunk ago) goes round with this barrier, and the one after it is asked for
        if (tid == 0) { s_ticket = next_ticket; next_ticket = atomicAdd(&ctl[0], 1); }
        __syncthreads();
        const int ticket_n = __builtin_amdgcn_readfirstlane(s_ticket);
        const Chunk nxt = chunk_of(ticket_n);

        // ---- the chunk's row maxima out, those of the chunks before it in
        const size_t unit = (size_t)bh * NC + ch;
        float pm = xr < R && xt < NT ? tmax[xr][xt] : -INFINITY;      // becomes the row's running maximum over the tiles
#pragma unroll
        for (int dd = 1; dd < 16; dd <<= 1) {
            const float up = __shfl_up(pm, dd, 16);
            if (xt >= dd) pm = fmaxf(pm, up);
        }
        if (nch > 1 && xt == 15 && xr < R)
            __hip_atomic_store(&cmax[unit * kDecRows + xr], (1ull << 32) | (unsigned long long)__float_as_uint(pm),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the maxima of the chunks in front: the one asked for early, and, on a path of its own (its loads wait for
        // everything in flight), whichever was not there yet and those of a chunk with more than 16 in front (bounded
        // polling; see the head of this file)
        float m_pred = -INFINITY;
        const bool early_wanted = xr < R && xt < ch, early_there = (v_early >> 32) != 0;
        if (early_wanted && early_there) m_pred = __uint_as_float((uint32_t)v_early);
        if (__builtin_amdgcn_ballot_w64(xr < R && ((early_wanted && !early_there) || xt + 16 < ch)) != 0 && xr < R) {
            for (int i = xt + (early_there ? 16 : 0); i < ch; i += 16) {
                const unsigned long long* src = &cmax[((size_t)bh * NC + i) * kDecRows + xr];
                unsigned long long v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int spins = 0; (v >> 32) == 0 && spins < spin_limit; ++spins) {
                    __builtin_amdgcn_s_sleep(8);
                    v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (v >> 32) m_pred = fmaxf(m_pred, __uint_as_float((uint32_t)v));
                else __hip_atomic_store(&ctl[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (int dd = 1; dd < 16; dd <<= 1) m_pred = fmaxf(m_pred, __shfl_xor(m_pred, dd, 16));
        if (xr < R && xt < NT) run[xr][xt] = fmaxf(m_pred, pm);
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
            if (t < NT) {
            const int k_t = key0 + 64 * t;
            RawKV<D> (&raw)[4] = rw[(it + 4) % 3];
            // P^F of the whole tile, four rows at a time
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                if (4 * ps < R) {
                    const int prow = min(4 * ps + pq, R - 1);
                    const float mrow = run[prow][t], ms = mrow * c;
                    const floatx4 sv = __builtin_bit_cast(floatx4, lds_read16_at(sbuf_ad + 4u * (uint32_t)(prow * CK + 64 * t + 4 * pj)));
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
                    const half2v sc = scales_of<D>(raw[2 * hh + sub], cur.ok[it] && k_t + 32 * hh + 16 * sub + cc < Lk);
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
            }
            // the slot of this tile's V part is free: the chunk's last item, then the next chunk's query rows (their
            // registers have been free since the scores) and its first K parts
            if (it == 0) { issue(cur, 7); load_q(nxt); }
            if (it == 1) issue(nxt, 2);
            if (it == 2) issue(nxt, 0);
            if (it == 3) issue(nxt, 1);
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
        } else {
            // several chunks: the partial sums go to memory for the kernel that adds them
            for (int e = tid; e < R * D; e += 256)
                part_o[unit * R * D + e] = (mbuf[e] + mbuf[R * D + e]) + (mbuf[2 * R * D + e] + mbuf[3 * R * D + e]);
            if (tid < R) {
                part_l[unit * kDecRows + tid] = (lsum_w[0][tid] + lsum_w[1][tid]) + (lsum_w[2][tid] + lsum_w[3][tid]);
                part_m[unit * kDecRows + tid] = run[tid][NT - 1];
            }
        }
        // (no barrier here: the next chunk's first half writes only its scores and tile maxima, which nobody reads any more,
        //  and everything else it writes lies behind its own barriers)
        cur = nxt;
        ticket = ticket_n;
    }
    // the loads that were issued for a chunk beyond the list land before the wave ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
                po[k] = part_o[u * R * D + e];
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
    size_t n = 256;                                                   // ticket counter, error word, number of chunks
    n += units * kDecRows * 8;                                         // row maxima with their tags
    n += units * kDecRows * 4 * 2;                                     // l and m of the partial sums
    n += units * R * D * 4;                                            // O of the partial sums (R rows each)
    n += units * kDecItemInts * 4;                                     // the list of chunks
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
    float* part_o = (float*)p;               p += units * R * D * 4;
    int* work = (int*)p;
    // the counters and the tagged row maxima are one run of ints from ctl on
    const size_t nz64 = ((unsigned char*)cmax - (unsigned char*)ctl) / 4 + units * kDecRows * 2;
    if (nz64 > 0x7FFFFFFFull) return -1;
    const int nz = (int)nz64;
    hipLaunchKernelGGL(decode_plan_kernel, dim3((nz + 255) / 256), dim3(256), 0, st, kv_lens, page_table, B, Hkv, R, D, CK, NC, max_pages, ctl, nz, work,
                       (uint16_t*)o, lse);
    if (hipGetLastError() != hipSuccess) return -1;
    const int cus = device_cu_count();
    const unsigned grid = (unsigned)min((size_t)2 * cus, units);
    const float c = 1.4426950408889634f / sqrtf((float)D);
#define AQ_DEC(DD, C) hipLaunchKernelGGL((decode_kernel<DD, C>), dim3(grid), dim3(256), 0, st, (const half_t*)qh, (const unsigned char*)cache, \
        num_pages, Hkv, Lq, R, CK, NC, spin_limit, ctl, work, cmax, part_o, part_l, part_m, \
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
