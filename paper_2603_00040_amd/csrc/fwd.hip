// Fused forward of Attn-QAT on gfx950: Alg. 1 (inference) and Alg. 2 (training).
//
// Work split: a workgroup of 8 waves owns 256 query rows of one head; each wave owns 32
// of them.  Key tiles of B_k = 64 keys are visited in increasing order; K and V^T tiles
// are copied global->LDS directly (global_load_lds, double buffered, XOR-swizzled rows)
// and shared by the eight waves.  Waves 0-3 and waves 4-7 run half an iteration apart
// (vector phase / matrix phase, separated by barriers).
//
// MFMA shapes (v_mfma_f32_32x32x16_f16, fp32 accumulate).  All operands are the
// dequantized NVFP4 values s*c, which fp16 represents exactly, so the products are those
// of Eq. 4 (BF16MM on fake-quantized operands == FP4MM of Eq. 3).
//   S^T[key, query]   = K^F (A, from LDS)   x  Q^F^T (B, registers)
//   O^T[d, query]    += V^F^T (A, from LDS) x  P-tilde^F^T (B, registers)
//   O'^T[d, query]   += V^F^T (same A)      x  P-tilde^T   (B, registers; training only)
// With S transposed, a lane owns ONE query row and 8+8 keys of every aligned group of 16
// keys: the row max, the row sum and the 16-key block max of phi(P-tilde) are register
// reductions plus one exchange between the two 32-lane halves, and the accumulator
// layout of S^T already is the B-operand layout of the P.V products (V^T is stored with
// the matching key permutation, see prep.hip).
#include "common.hpp"
#include "kernels.hpp"

namespace aq {

template <int D>
struct FwdSmem {
    half_t k[2][64 * D];      // K tile [key][d], 16-byte chunks XOR-swizzled inside a row
    half_t v[2][D * 64];      // V^T tile [d][key], likewise
};

// PQ, the format of P-tilde in the P V product: 0 NVFP4, 1 MX, 2 NVFP4 with the two-level row factor,
// 3 bf16 with V left in bf16 as well (the mixed recipe "NVFP4 Q K^T, BF16 P V" of Sec. 2.5; the tile buffer of V^T then
// holds bf16 bit patterns and the P V products are bf16 MFMAs; inference only).
// VARLEN (serving): every sequence b has its own number of keys kv_lens[b] (read here, on the device), the copies of K and V^T
// are laid out for Lkp positions per head, and the L query rows are the LAST L positions of their sequence: under the causal
// mask query i sees keys 0 .. kv_lens[b] - L + i (a chunk of a prefill; needs kv_lens[b] >= L).
template <int D, bool TRAIN, bool CAUSAL, bool DUMP, int PQ, bool VARLEN = false>
__global__ __launch_bounds__(512, 2) void fwd_kernel(
    const half_t* __restrict__ Qh, const half_t* __restrict__ Kh, const half_t* __restrict__ Vt,
    uint16_t* __restrict__ O, float* __restrict__ lse, float* __restrict__ Ohp,
    int L, int Lp, int Hq, int G, float c /* log2(e)/sqrt(d) */, int dump_row0, float* __restrict__ pdump,
    int Lkp_arg, const int* __restrict__ kv_lens, const uint32_t* __restrict__ Qsc)
{
    // PQ == 1 (MX): S = Q^F K^F^T comes from the E2M1 codes and E8M0 scales by v_mfma_scale_f32_32x32x64_f8f6f4 (a quarter of
    // the matrix time of the 16-bit products, a quarter of the K bytes through LDS).  Qh then holds the Q operands of that
    // instruction (64 d per step: lane (row, half) has d-slots 64 ks + 32 half .. + 31 of its row) with one dword of scale
    // bytes per lane in Qsc, and Kh the K records of mx_ktrain_rec_bytes(D) bytes per key tile.  The accumulator layout is
    // that of the 16-bit products, so everything after the scores is unchanged (O and O' stay 16-bit products: O' needs the
    // un-quantized P-tilde, which is no operand of that instruction).
    constexpr bool MXS = PQ == 1;
    constexpr int KSM = D / 64, KREC = mx_ktrain_rec_bytes(D);
    typedef int int8v __attribute__((ext_vector_type(8)));
    constexpr int DS = D / 16;      // contraction steps of S
    constexpr int MB = D / 32;      // 32-row blocks of O^T
    constexpr int KCH = D / 8;      // 16-byte chunks per K row
    constexpr int KLD = KCH / 8;    // 1 KiB wave-loads per wave for the K tile (8 waves)
    constexpr int VLD = D / 64;     // ... for the V^T tile
    extern __shared__ __align__(256) unsigned char smem_raw[];   // the XORs of address bits 5..7 commute with adding this base
    FwdSmem<D>& sm = *reinterpret_cast<FwdSmem<D>*>(smem_raw);

    // Work items: a tile of 256 query rows of one head.  Without a mask a workgroup takes one.  Under a causal mask tile qt
    // visits 4 qt + 4 key tiles, so a workgroup takes a pair, tile nqt - 1 - p and then tile p: every workgroup then does
    // the same amount of work (no tail of long tiles at the end of a head) and there are half as many workgroups, each of
    // which costs the CU a fixed 20 - 30 us of start-up and wind-down that nothing overlaps at one workgroup per CU.
    const int nqt = (Lp + 255) / 256;
    const int per_head = CAUSAL ? (nqt + 1) / 2 : nqt;
    int bh, qt0;
    head_tile_of_block(blockIdx.x, gridDim.x / per_head, per_head, bh, qt0);
    const int nitems = (CAUSAL && nqt - 1 - qt0 != qt0) ? 2 : 1;
    const int b = bh / Hq, h = bh % Hq;
    const int bhkv = b * (Hq / G) + h / G;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);        // scalar: LDS destinations and branches use it
    const bool late = wave >= 4;                         // the group that runs one phase behind
    // keys of this sequence, row stride of the K / V^T copies, and how far the causal diagonal is shifted
    const int Lk = VARLEN ? max(1, min(kv_lens[b], Lkp_arg)) : L;
    const int Lkp = VARLEN ? Lkp_arg : Lp;
    const int off = (VARLEN && CAUSAL) ? max(0, Lk - L) : 0;
    const int nkt_all = (Lk + 63) / 64;

    for (int item = 0; item < nitems; ++item) {
    // (the lane number is taken afresh for every item and made opaque: everything formed from it would otherwise be kept
    //  in registers, or rather in scratch, across the key loop for the sake of the second item)
    uint32_t lane_i = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(lane_i));
    const int lane = (int)lane_i, ln = lane & 31, hf = lane >> 5;

    // Chunk c of row r sits at chunk c ^ key(r), so an operand's byte offset is (per-lane constant) XOR
    // (compile-time constant): K rows  k_rd ^ (ds << 5),  V^T rows  v_rd ^ (ks << 5); 32 more rows and
    // the other buffer are constant distances.
    const int k_rd = 2 * swz_elem<KCH>(ln, 8 * hf);
    const int v_rd = 2 * swz_elem<8>(ln, 8 * hf);
    const unsigned char* kbase = reinterpret_cast<const unsigned char*>(&sm.k[0][0]);
    const unsigned char* vbase = reinterpret_cast<const unsigned char*>(&sm.v[0][0]);

    // direct-to-LDS tile loads: wave-uniform tile base + this lane's byte offset inside the tile
    uint32_t k_ld[KLD], v_ld[VLD];
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
        const int slot = 64 * (wave * KLD + i) + lane, r = slot / KCH, pc = slot % KCH;
        k_ld[i] = 2u * (uint32_t)(r * D + 8 * swz<KCH>(r, pc));
    }
#pragma unroll
    for (int i = 0; i < VLD; ++i) {
        const int slot = 64 * (wave * VLD + i) + lane, r = slot / 8, pc = slot % 8;
        v_ld[i] = 2u * ((uint32_t)r * (uint32_t)Lkp + 8u * (uint32_t)swz<8>(r, pc));
    }
    const half_t* k_head = Kh + (size_t)bhkv * Lkp * D;      // [key][d]
    const half_t* v_head = Vt + (size_t)bhkv * D * Lkp;      // [d][key]
    const unsigned char* k_recs = reinterpret_cast<const unsigned char*>(Kh) + (size_t)bhkv * (Lkp / 64) * KREC;
    auto issue_k = [&](int buf, int jt) __attribute__((always_inline)) {
        if constexpr (MXS) {      // a record is KREC / 1024 wave copies of 1 KiB
            if (wave < KREC / 1024)
                async_copy16(k_recs + (size_t)jt * KREC, (uint32_t)(wave * 1024 + lane * 16), reinterpret_cast<unsigned char*>(&sm.k[buf][0]) + wave * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < KLD; ++i) async_copy16(k_head + (size_t)jt * (64 * D), k_ld[i], &sm.k[buf][512 * (wave * KLD + i)]);
        }
    };
    auto issue_v = [&](int buf, int jt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < VLD; ++i) async_copy16(v_head + (size_t)jt * 64, v_ld[i], &sm.v[buf][512 * (wave * VLD + i)]);
    };

    const int qt = CAUSAL ? (item == 0 ? nqt - 1 - qt0 : qt0) : qt0;
    const int row0_w = qt * 256 + wave * 32;
    const bool has_rows = row0_w < Lp;                   // false only in the last tile of a head
    const int q_row = row0_w + ln;

    // Q^F operand: this lane's query row, d-slots 16*ds + 8*hf .. +7
    half8 qreg[MXS ? 1 : DS];
    uint4v qop[MXS ? KSM : 1];
    uint32_t qs = 0u;
    if constexpr (MXS) {
        const size_t grp = (size_t)bh * (Lp / 32) + ((has_rows ? row0_w : 0) >> 5);
        const unsigned char* qo = reinterpret_cast<const unsigned char*>(Qh);
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) qop[ks] = *reinterpret_cast<const uint4v*>(qo + ((grp * KSM + ks) * 64 + lane) * 16);
        qs = Qsc[grp * 64 + lane];
    } else {
        const half_t* qp = Qh + ((size_t)bh * Lp + (has_rows ? q_row : 0)) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) qreg[ds] = *reinterpret_cast<const half8*>(qp + 16 * ds);
    }
    const int nkt = CAUSAL ? min((qt * 256 + 255 + off) / 64 + 1, nkt_all) : nkt_all;     // key tiles this item visits
    const int wave_qmax = row0_w + 31 + off;             // the last key that a row of this wave sees

    floatx16 o[MB], op[TRAIN ? MB : 1];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { o[mb][i] = 0.0f; if constexpr (TRAIN) op[mb][i] = 0.0f; }
    }
    float m = -INFINITY, lsum = 0.0f;     // lsum: this half-wave's part of l (same alpha in both halves)
    float s1_prev = 1.0f, s1_cur = 1.0f;  // two-level P-tilde: the row factor O is currently expressed in, and this tile's
    floatx16 s[2];                        // S^T of the current tile, then P-tilde
#pragma unroll
    for (int i = 0; i < 16; ++i) { s[0][i] = 0.0f; s[1][i] = 0.0f; }

    // ---- S^T = K^F Q^F^T of one tile.  A wave sustains about one 1 KiB LDS read per 40 cycles and the
    // read latency is ~130 cycles, so the K operands are read RING steps ahead of the MFMA that consumes
    // them (the scheduling groups keep the compiler from sinking them).
    auto scores = [&](int buf) __attribute__((always_inline)) {
        if constexpr (MXS) {
            const uint32_t rec = lds_addr_of(kbase) + (uint32_t)(buf * (int)sizeof(sm.k[0]));
            const uint32_t ksc = *(const __attribute__((address_space(3))) uint32_t*)(uintptr_t)(rec + 2 * KSM * 1024 + lane * 4);
            uint4v a[2][KSM];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int ks = 0; ks < KSM; ++ks) a[kb][ks] = lds_read16_at(rec + (uint32_t)(((kb * KSM + ks) * 64 + lane) * 16));
            auto as8 = [](const uint4v& x) __attribute__((always_inline)) -> int8v {
                int8v r = {(int)x[0], (int)x[1], (int)x[2], (int)x[3], 0, 0, 0, 0};
                return r;
            };
            const floatx16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
            // (format codes 4, 4: both operands E2M1; the scale operands are a dword of four bytes and the index of the byte)
            s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0][0]), as8(qop[0]), zero, 4, 4, 0, ksc, 0, qs);
            s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1][0]), as8(qop[0]), zero, 4, 4, KSM, ksc, 0, qs);
            if constexpr (KSM == 2) {
                s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0][1]), as8(qop[1]), s[0], 4, 4, 1, ksc, 1, qs);
                s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1][1]), as8(qop[1]), s[1], 4, 4, 3, ksc, 1, qs);
            }
            mfma_scale_settle(s[0], s[1]);
            return;
        }
        // per-lane offset of this tile, opaque to the compiler: it would otherwise hoist every
        // (offset ^ constant) out of the loop and pay for it with registers
        int k_it = k_rd + buf * (int)sizeof(sm.k[0]) + (int)lds_addr_of(kbase);
        asm volatile("" : "+v"(k_it));
        auto k_opnd = [&](int i) __attribute__((always_inline)) -> half8 {
            return __builtin_bit_cast(half8, lds_read16_at((uint32_t)((k_it ^ ((i >> 1) << 5)) + (i & 1) * (32 * D * 2))));
        };
        constexpr int NS = 2 * DS, RING = 6;
        half8 ring[RING];
#pragma unroll
        for (int i = 0; i < RING; ++i) ring[i] = k_opnd(i);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
#pragma unroll
        for (int i = 0; i < NS; ++i) {                  // step i: ds = i / 2, kb = i % 2
            const half8 a = ring[i % RING];
            if (i + RING < NS) ring[i % RING] = k_opnd(i + RING);
            s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[i >> 1], s[i & 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + RING < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    // ---- prologue: K(0), V(0), K(1) land, then every wave computes its S of tile 0
    issue_k(0, 0);
    issue_v(0, 0);
    if (nkt > 1) issue_k(1, 1);
    // The Q registers must have arrived BEFORE the loop: a load still pending at loop entry makes the
    // compiler wait for all vector-memory traffic at the first product of every iteration.
    if constexpr (MXS) {
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) asm volatile("" : "+v"(qop[ks]));
        asm volatile("" : "+v"(qs));
    } else {
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) asm volatile("" : "+v"(qreg[ds]));
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (has_rows) scores(0);
    if (late) __builtin_amdgcn_s_barrier();              // one phase behind from here on

    // Two phases per key tile, separated by barriers; waves 0-3 are in the vector phase while waves
    // 4-7 are in the matrix phase and vice versa, so every SIMD holds one wave of each kind:
    //   vector phase j:  mask, online softmax, block scales of phi(P-tilde)         (no MFMA, no LDS)
    //   matrix phase j:  O, O' += V^F^T P(j) with the FP4 round trip of P-tilde in between;  S(j+1)
    // (The MFMAs of one wave do not overlap with the vector instructions of ANOTHER wave on this
    // hardware, only with its own; what this arrangement buys, measured, is that the matrix stream
    // runs at raised priority against a pure vector stream and that a tile copy serves 256 rows.)
    // Tile traffic: K(j+2) and V(j+1) are requested at the start of matrix phase j into the buffers
    // whose last readers (matrix phase j-1 of either group) are two barriers back.
    // ---- vector phase of one key tile: mask, online softmax, block scales of phi(P-tilde)  (no MFMA, no LDS)
    auto vector_phase = [&](int j, float (&bsc)[4], float (&binv)[4]) __attribute__((always_inline)) {
        const int k0 = j * 64;
        // mask: keys beyond L, and keys after the query when causal
        const bool need_mask = (k0 + 64 > Lk) || (CAUSAL && k0 + 63 > row0_w + off);
        if (__builtin_expect(need_mask, 0)) {
            const int klim = CAUSAL ? min(Lk - 1, q_row + off) : Lk - 1;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = k0 + 32 * kb + 8 * (i >> 2) + 4 * hf + (i & 3);
                    if (key > klim) s[kb][i] = -INFINITY;
                }
        }
        // online softmax (Alg. 2: m_new, alpha, P-tilde, l).  Four interleaved chains each: a single
        // chain of 32 dependent max / add instructions would run at the instruction latency.
        // The maxima are taken on S: one per group of 16 keys (registers 8g..8g+7 of both halves), the tile's row
        // maximum from those four.  exp2 of a group's largest score, by the same instructions on the same inputs as
        // that element's P-tilde, then is the group's largest P-tilde, which the block scale of phi needs below.
        float mt, gmax[4];
        if constexpr (PQ == 1 || PQ == 3) {
            float mp[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) mp[t] = max_nc(s[0][t], s[1][t]);
#pragma unroll
            for (int i = 4; i < 16; ++i) mp[i & 3] = max_nc(max_nc(mp[i & 3], s[0][i]), s[1][i]);
            mt = xhalf_max(max_nc(max_nc(mp[0], mp[1]), max_nc(mp[2], mp[3])));
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const floatx16& sv = s[ks >> 1];
                const int b0 = 8 * (ks & 1);
                const float a0 = max_nc(max_nc(sv[b0], sv[b0 + 1]), sv[b0 + 2]);
                const float a1 = max_nc(max_nc(sv[b0 + 3], sv[b0 + 4]), sv[b0 + 5]);
                gmax[ks] = max_nc(max_nc(a0, a1), max_raw(sv[b0 + 6], sv[b0 + 7]));
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) gmax[ks] = xhalf_max(gmax[ks]);
            mt = max_nc(max_nc(gmax[0], gmax[1]), max_nc(gmax[2], gmax[3]));
        }
        const float mnew = max_nc(m, mt);
        const float alpha = __builtin_amdgcn_exp2f((m - mnew) * c);
        const float ms = mnew * c;
        m = mnew;
        float rp[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -ms));
                if (kb == 0 && i < 4) rp[i] = s[kb][i];
                else                  rp[i & 3] += s[kb][i];
            }
        lsum = lsum * alpha + ((rp[0] + rp[1]) + (rp[2] + rp[3]));          // un-quantized P-tilde
        // rescale: exact no-op unless some row of this wave moved its maximum (rare after the
        // first tiles), so it lives on the cold path
        float inv1 = 1.0f;
        if constexpr (PQ == 2) {
            // Two-level quantization of P-tilde (Sec. 2.1): the row of this tile is divided by s1, the smallest power
            // of two with 2688 s1 >= max(row maximum, 2^-24), before the NVFP4 blocks.  The row maximum is exp2 of the
            // tile's largest score, the same instructions on the same inputs as that element's P-tilde.
            // O is kept in units of the current s1 (its products use P-tilde / s1, which fp16 holds exactly whatever
            // the magnitude of the row), so it is re-based on every tile; O' only needs alpha.
            const float base = fmaxf(__builtin_amdgcn_exp2f(fmaf(mt, c, -ms)), 5.9604644775390625e-08f);
            const uint32_t e1 = ((__float_as_uint(base) + 0x0057FFFFu) >> 23) - 11u;      // 2688 = 1.3125 * 2^11
            s1_cur = __uint_as_float(e1 << 23);
            inv1 = __uint_as_float((254u - e1) << 23);
            const float f = alpha * s1_prev * inv1;
            s1_prev = s1_cur;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[mb][i] *= f;
            if constexpr (TRAIN) {
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0, 0)) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) op[mb][i] *= alpha;
                }
            }
        } else if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0, 0)) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) { o[mb][i] *= alpha; if constexpr (TRAIN) op[mb][i] *= alpha; }
        }
        if constexpr (PQ == 3) return;      // bf16 P-tilde has no block scales
        if constexpr (PQ == 1) {
            // MX format: one power-of-two scale per 32 keys = all 16 registers of s[kb] in both halves;
            // the two 16-key groups of a block share it
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const floatx16& sv = s[kb];
                float a4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) a4[t] = fmaxf(fmaxf(sv[t], sv[4 + t]), fmaxf(sv[8 + t], sv[12 + t]));
                const uint32_t byte = e8m0_of_amax(xhalf_max(fmaxf(fmaxf(a4[0], a4[1]), fmaxf(a4[2], a4[3]))));
                bsc[2 * kb] = bsc[2 * kb + 1] = e8m0_as_f32(byte);
                binv[2 * kb] = binv[2 * kb + 1] = e8m0_inverse_as_f32(byte);
            }
            return;
        }
        // block scales of phi(P-tilde) for the four 16-key groups of the tile (keys of a group =
        // registers 8g..8g+7 of both halves), as four independent chains
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) bsc[ks] = __builtin_amdgcn_exp2f(fmaf(gmax[ks], c, -ms));
        // (two-level: the block maxima of P-tilde / s1 are at most 2688 (1 + 2^-23), whose sixth rounds to 448, the largest scale)
        if constexpr (PQ == 0) {
            // RNE_E4M3(amax / 6) by the hardware conversion (OCP E4M3, round to nearest even, subnormals kept; two values
            // per instruction) and back: the same values as rne_e4m3_grid in a quarter of the instructions.
            // P-tilde <= 1: no saturation
            typedef short short2v __attribute__((ext_vector_type(2)));
            short2v pk = {0, 0};
            pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, bsc[0] * (1.0f / 6.0f), bsc[1] * (1.0f / 6.0f), 1.0f, false);
            pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, bsc[2] * (1.0f / 6.0f), bsc[3] * (1.0f / 6.0f), 1.0f, true);
            const uint32_t w = __builtin_bit_cast(uint32_t, pk);
            bsc[0] = __builtin_amdgcn_cvt_scalef32_f32_fp8(w, 1.0f, 0);
            bsc[1] = __builtin_amdgcn_cvt_scalef32_f32_fp8(w, 1.0f, 1);
            bsc[2] = __builtin_amdgcn_cvt_scalef32_f32_fp8(w, 1.0f, 2);
            bsc[3] = __builtin_amdgcn_cvt_scalef32_f32_fp8(w, 1.0f, 3);
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bsc[ks] = rne_e4m3_grid((bsc[ks] * inv1) * (1.0f / 6.0f));
        }
        // reciprocals.  A scale of 0: P^F is 0 whatever the codes are (the dequantization multiplies by the scale), so
        // any finite factor serves; 512 = 1 / (smallest non-zero scale) keeps the quotients finite.
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) binv[ks] = fminf(__builtin_amdgcn_rcpf(bsc[ks]), 512.0f) * inv1;
    };
    // ---- matrix phase of one key tile: O, O' += V^F^T P with the FP4 round trip of P-tilde in between
    auto matrix_phase = [&](int j, const float (&bsc)[4], const float (&binv)[4]) __attribute__((always_inline)) {
        const int k0 = j * 64;
        (void)k0;
        // per 16 keys: phi^-1(phi(P-tilde)), then O^T += V^F^T P-tilde^F^T and O'^T += V^F^T P-tilde^T
        // (an LDS address as an integer: pointer arithmetic on the dynamic LDS symbol costs an add per read)
        int v_it = v_rd + (j & 1) * (int)sizeof(sm.v[0]) + (int)lds_addr_of(vbase);
        asm volatile("" : "+v"(v_it));
        struct QState { uint32_t c01, c23; };
        float pfv[DUMP ? 8 : 1];
        // the FP4 round trip of one group of 16 keys, cut into four parts of a few instructions
        auto q_part = [&](int ks, int part, QState& st, uint4v& bq, uint4v& bu) __attribute__((always_inline)) {
            const int b0 = 8 * (ks & 1);
            const floatx16& sv = s[ks >> 1];
            if constexpr (PQ == 3) {
                // bf16 P-tilde: one rounding (nearest even), no codes and no scales
                if (part == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) bq[i] = pack_bf16x2_cvt(sv[b0 + 2 * i], sv[b0 + 2 * i + 1]);
                    if constexpr (DUMP) {
                        if (q_row >= dump_row0 && q_row < dump_row0 + 128 && q_row < L) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const int key = k0 + 32 * (ks >> 1) + 16 * (ks & 1) + 8 * (i >> 2) + 4 * hf + (i & 3);
                                if (key < L)
                                    pdump[((size_t)bh * 128 + (q_row - dump_row0)) * L + key] =
                                        __uint_as_float((i & 1) ? (bq[i >> 1] & 0xFFFF0000u) : (bq[i >> 1] << 16));
                            }
                        }
                    }
                }
                return;
            }
            const float inv = binv[ks];
            if (part == 0) {
                // (the conversion replaces one byte of its first operand; bytes 2 and 3 of the code registers are never
                //  read, so any register that is live anyway serves and none has to be cleared)
                st.c01 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(__float_as_uint(inv), sv[b0] * inv, sv[b0 + 1] * inv, 1.0f, 0);
                st.c23 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(__float_as_uint(inv), sv[b0 + 4] * inv, sv[b0 + 5] * inv, 1.0f, 0);
            } else if (part == 1) {
                st.c01 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(st.c01, sv[b0 + 2] * inv, sv[b0 + 3] * inv, 1.0f, 1);
                st.c23 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(st.c23, sv[b0 + 6] * inv, sv[b0 + 7] * inv, 1.0f, 1);
            } else if (part == 2) {
                const half2v sc2 = __builtin_bit_cast(half2v, pack_f16x2(bsc[ks], bsc[ks]));
                uint32_t w[4];
                w[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c01, 1.0f, 0) * sc2);
                w[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c01, 1.0f, 1) * sc2);
                w[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c23, 1.0f, 0) * sc2);
                w[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c23, 1.0f, 1) * sc2);
                bq[0] = w[0]; bq[1] = w[1]; bq[2] = w[2]; bq[3] = w[3];
                if constexpr (DUMP) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const half2v pr = __builtin_bit_cast(half2v, w[i]);
                        pfv[2 * i] = (float)pr[0]; pfv[2 * i + 1] = (float)pr[1];
                    }
                    if (q_row >= dump_row0 && q_row < dump_row0 + 128 && q_row < L) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int key = k0 + 32 * (ks >> 1) + 16 * (ks & 1) + 8 * (i >> 2) + 4 * hf + (i & 3);
                            if (key < L)
                                pdump[((size_t)bh * 128 + (q_row - dump_row0)) * L + key] = PQ == 2 ? pfv[i] * s1_cur : pfv[i];
                        }
                    }
                }
            } else if constexpr (TRAIN) {
#pragma unroll
                for (int i = 0; i < 4; ++i) bu[i] = pack_f16x2(sv[b0 + 2 * i], sv[b0 + 2 * i + 1]);
            }
        };
        // A wave issues in order: a block of MFMAs followed by a block of vector instructions leaves the
        // vector ALU idle while the MFMAs queue up.  So the parts of step ks+1 follow the products of
        // step ks one by one (scheduling fences keep the compiler from regrouping them); a V^T operand
        // register is reloaded for step ks+1 as soon as its last product of step ks has issued.
        half8 av[MB];
        uint4v bq[2], bu[2];
        QState st;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            av[mb] = __builtin_bit_cast(half8, lds_read16_at((uint32_t)(v_it + mb * (32 * 64 * 2))));
#pragma unroll
        for (int part = 0; part < 4; ++part) q_part(0, part, st, bq[0], bu[0]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            const half8 bqh = __builtin_bit_cast(half8, bq[cur]);
            const half8 buh = __builtin_bit_cast(half8, bu[cur]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if constexpr (!DUMP) __builtin_amdgcn_sched_barrier(0);
                if constexpr (PQ == 3)
                    o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[mb]), __builtin_bit_cast(bf16x8, bqh), o[mb], 0, 0, 0);
                else
                    o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], bqh, o[mb], 0, 0, 0);
                if constexpr (TRAIN) {
                    if constexpr (!DUMP) __builtin_amdgcn_sched_barrier(0);
                    op[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], buh, op[mb], 0, 0, 0);
                }
                if (ks < 3) {
#pragma unroll
                    for (int part = (4 * mb) / MB; part < (4 * (mb + 1)) / MB; ++part) q_part(ks + 1, part, st, bq[nxt], bu[nxt]);
                    av[mb] = __builtin_bit_cast(half8, lds_read16_at((uint32_t)((v_it ^ ((ks + 1) << 5)) + mb * (32 * 64 * 2))));
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        };
    // the tile copies of matrix phase j
    auto request_tiles = [&](int j) __attribute__((always_inline)) {
        if (j + 2 < nkt) issue_k(j & 1, j + 2);
        if (j + 1 < nkt) issue_v((j + 1) & 1, j + 1);
    };

    // Under a causal mask the workgroup's first 4 qt + 1 key tiles are visible to every one of its waves (the tile that
    // starts at the workgroup's first row included; rows inside it are masked in the vector phase), and only the last
    // three have waves that skip.  The two kinds of tile get loops of their own: the form with the skipping branch
    // schedules markedly worse (17 % slower on tiles where nobody skips), so it only runs where somebody does.
    const int j_all = CAUSAL ? min(nkt, (qt * 256 + 31 + off) / 64 + 1) : nkt;
    for (int j = 0; j < j_all; ++j) {
        const int k0 = j * 64;
        float bsc[4], binv[4];
        if (has_rows) vector_phase(j, bsc, binv);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_s_setprio(1);    // the MFMA stream is the scarce one: it wins issue conflicts
        request_tiles(j);
        if (has_rows) matrix_phase(j, bsc, binv);
        // S of the next tile (its P-tilde predecessor in the same registers has been consumed above)
        if (has_rows && j + 1 < nkt && (!CAUSAL || k0 + 64 <= wave_qmax)) scores((j + 1) & 1);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_s_waitcnt(0);        // this wave's parts of K(j+2) and V(j+1) are in LDS
        __builtin_amdgcn_s_barrier();
    }
    if constexpr (CAUSAL) {
        for (int j = j_all; j < nkt; ++j) {
            const int k0 = j * 64;
            const bool active = has_rows && k0 <= wave_qmax;          // wave-uniform
            // Waves skip the tiles above the diagonal.  The whole tile sits in one branch, with a barrier on
            // either path: written as two branches around a common barrier, the softmax state looks live to
            // the compiler on the skipping path and the kernel spills.
            if (active) {
                float bsc[4], binv[4];
                vector_phase(j, bsc, binv);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_s_setprio(1);
                request_tiles(j);
                matrix_phase(j, bsc, binv);
            } else {
                __builtin_amdgcn_s_barrier();
                request_tiles(j);
            }
            if (has_rows && j + 1 < nkt && k0 + 64 <= wave_qmax) scores((j + 1) & 1);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_s_barrier();
        }
    }
    if (!late) __builtin_amdgcn_s_barrier();             // pairs with the late group's extra barrier

    // ---- epilogue: O /= l, O' /= l, L = m + log l
    const float l = xhalf_sum(lsum);
    const float inv_l = 1.0f / l;
    const float inv_lo = PQ == 2 ? s1_prev * inv_l : inv_l;      // O leaves the units of the last row factor
    if (q_row < L) {
        const size_t row = (size_t)bh * L + q_row;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int d0 = 32 * mb + 8 * t + 4 * hf;
                uint2v w;
                w[0] = pack_bf16x2_rne(o[mb][4 * t] * inv_lo, o[mb][4 * t + 1] * inv_lo);
                w[1] = pack_bf16x2_rne(o[mb][4 * t + 2] * inv_lo, o[mb][4 * t + 3] * inv_lo);
                *reinterpret_cast<uint2v*>(O + row * D + d0) = w;
                if constexpr (TRAIN) {
                    floatx4 f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[e] = op[mb][4 * t + e] * inv_l;
                    *reinterpret_cast<floatx4*>(Ohp + row * D + d0) = f;
                }
            }
        if (hf == 0) lse[row] = m * (c * 0.6931471805599453f) + logf(l);   // m is in raw q.k units
    }
    // (a second item may overwrite the tile buffers at once: every wave's last read of them lies before a barrier that
    //  all eight waves have passed by now)
    }
}

template <int D, bool TRAIN, bool CAUSAL, bool DUMP, int PQ, bool VARLEN = false>
static int launch_t(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int L,
                    void* o, float* lse, float* o_hp, int dump_row0, float* p_dump, hipStream_t st,
                    int Lkp = 0, const int* kv_lens = nullptr, const void* qsc = nullptr)
{
    if (PQ == 1 && !qsc) return -1;
    const int Lp = round_up(L, kRowPad);
    const int nqt = (Lp + 255) / 256;
    const int per_head = CAUSAL ? (nqt + 1) / 2 : nqt;         // under a causal mask a workgroup takes a long and a short tile
    const size_t smem = sizeof(FwdSmem<D>);
    auto kern = fwd_kernel<D, TRAIN, CAUSAL, DUMP, PQ, VARLEN>;
    static unsigned long long lds_set = 0;          // one per instantiation
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return -1;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq * per_head)), dim3(512), smem, st,
                       (const half_t*)qh, (const half_t*)kh, (const half_t*)vt, (uint16_t*)o, lse, o_hp,
                       L, Lp, Hq, Hq / Hkv, c, dump_row0, p_dump, Lkp, kv_lens, (const uint32_t*)qsc);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D, int PQ>
static int launch_d(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int L,
                    bool causal, bool train, void* o, float* lse, float* o_hp,
                    int dump_row0, float* p_dump, hipStream_t st, const void* qsc)
{
    if (p_dump) {
        return causal ? launch_t<D, false, true, true, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, dump_row0, p_dump, st, 0, nullptr, qsc)
                      : launch_t<D, false, false, true, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, dump_row0, p_dump, st, 0, nullptr, qsc);
    }
    if constexpr (PQ != 3) {
        if (train) {
            return causal ? launch_t<D, true, true, false, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st, 0, nullptr, qsc)
                          : launch_t<D, true, false, false, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st, 0, nullptr, qsc);
        }
    }
    return causal ? launch_t<D, false, true, false, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st, 0, nullptr, qsc)
                  : launch_t<D, false, false, false, PQ>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st, 0, nullptr, qsc);
}

int launch_fwd(const void* qh, const void* kh, const void* vt,
               int B, int Hq, int Hkv, int L, int D, bool causal, bool train, int p_quant,
               void* o, float* lse, float* o_hp, int dump_row0, float* p_dump, hipStream_t st, const void* qsc)
{
#define AQ_FWD(DD, PQ) launch_d<DD, PQ>(qh, kh, vt, B, Hq, Hkv, L, causal, train, o, lse, o_hp, dump_row0, p_dump, st, qsc)
    if (p_quant == 3 && train) return -1;           // the bf16 P V recipe has no backward
    if (D == 128) return p_quant == 1 ? AQ_FWD(128, 1) : p_quant == 2 ? AQ_FWD(128, 2) : p_quant == 3 ? AQ_FWD(128, 3) : AQ_FWD(128, 0);
    if (D == 64)  return p_quant == 1 ? AQ_FWD(64, 1) : p_quant == 2 ? AQ_FWD(64, 2) : p_quant == 3 ? AQ_FWD(64, 3) : AQ_FWD(64, 0);
#undef AQ_FWD
    return -1;
}

// Alg. 1 for sequences of different lengths: the last Lq positions of every sequence as queries, kv_lens[b] keys, K and V^T
// copies laid out for Lkp positions per head (a multiple of 64).
int launch_fwd_varlen(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int Lq, int Lkp, int D, bool causal,
                      const int* kv_lens, void* o, float* lse, hipStream_t st)
{
    if (!kv_lens || Lkp < 64 || Lkp % 64) return -1;
#define AQ_FWDV(DD, C) launch_t<DD, false, C, false, 0, true>(qh, kh, vt, B, Hq, Hkv, Lq, o, lse, nullptr, 0, nullptr, st, Lkp, kv_lens)
    if (D == 128) return causal ? AQ_FWDV(128, true) : AQ_FWDV(128, false);
    if (D == 64)  return causal ? AQ_FWDV(64, true) : AQ_FWDV(64, false);
#undef AQ_FWDV
    return -1;
}

}  // namespace aq
