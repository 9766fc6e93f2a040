// Fused forward of Attn-QAT on gfx950: Alg. 1 (inference) and Alg. 2 (training).
//
// Work split: a workgroup of 4 waves owns 128 query rows of one head; each wave owns 32
// of them.  Key tiles of B_k = 64 keys are visited in increasing order; K and V^T tiles
// are copied global->LDS directly (global_load_lds, double buffered, XOR-swizzled rows)
// and shared by the four waves.
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

template <int D, bool TRAIN, bool CAUSAL, bool DUMP>
__global__ __launch_bounds__(256, 2) void fwd_kernel(
    const half_t* __restrict__ Qh, const half_t* __restrict__ Kh, const half_t* __restrict__ Vt,
    uint16_t* __restrict__ O, float* __restrict__ lse, float* __restrict__ Ohp,
    int L, int Lp, int Hq, int G, float c /* log2(e)/sqrt(d) */, int dump_row0, float* __restrict__ pdump)
{
    constexpr int DS = D / 16;      // contraction steps of S
    constexpr int MB = D / 32;      // 32-row blocks of O^T
    constexpr int KCH = D / 8;      // 16-byte chunks per K row
    constexpr int KLD = KCH / 4;    // 1 KiB wave-loads per wave for the K tile
    constexpr int VLD = D / 32;     // ... for the V^T tile
    extern __shared__ __align__(16) unsigned char smem_raw[];
    FwdSmem<D>& sm = *reinterpret_cast<FwdSmem<D>*>(smem_raw);

    const int nqt = Lp / 128;
    const int bh = blockIdx.x / nqt;
    int qt = blockIdx.x % nqt;
    if (CAUSAL) qt = nqt - 1 - qt;                       // longest rows first
    const int b = bh / Hq, h = bh % Hq;
    const int bhkv = b * (Hq / G) + h / G;
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // scalar: LDS destinations and branches use it
    const int q_row = qt * 128 + wave * 32 + ln;

    // Q^F operand: this lane's query row, d-slots 16*ds + 8*hf .. +7
    half8 qreg[DS];
    {
        const half_t* qp = Qh + ((size_t)bh * Lp + q_row) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) qreg[ds] = *reinterpret_cast<const half8*>(qp + 16 * ds);
    }

    const int nkt_all = (L + 63) / 64;
    const int nkt = CAUSAL ? min(2 * qt + 2, nkt_all) : nkt_all;     // tiles this workgroup visits
    const int wave_qmax = qt * 128 + wave * 32 + 31;

    // LDS element offsets of this lane's operand reads (buffer 0, row block 0); the row blocks
    // kb / mb add compile-time constants because a row's swizzle key survives adding 32 rows.
    // Chunk c of row r sits at chunk c ^ key(r), so an operand's byte offset is (per-lane constant) XOR
    // (compile-time constant): K rows  k_rd ^ (ds << 5),  V^T rows  v_rd ^ (ks << 5).
    const int k_rd = 2 * swz_elem<KCH>(ln, 8 * hf);
    const int v_rd = 2 * swz_elem<8>(ln, 8 * hf);

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
        v_ld[i] = 2u * ((uint32_t)r * (uint32_t)Lp + 8u * (uint32_t)swz<8>(r, pc));
    }
    const half_t* k_head = Kh + (size_t)bhkv * Lp * D;      // [key][d]
    const half_t* v_head = Vt + (size_t)bhkv * D * Lp;      // [d][key]
    auto issue_tile = [&](int buf, int jt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < KLD; ++i) async_copy16(k_head + (size_t)jt * (64 * D), k_ld[i], &sm.k[buf][512 * (wave * KLD + i)]);
#pragma unroll
        for (int i = 0; i < VLD; ++i) async_copy16(v_head + (size_t)jt * 64, v_ld[i], &sm.v[buf][512 * (wave * VLD + i)]);
    };

    floatx16 o[MB], op[TRAIN ? MB : 1];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { o[mb][i] = 0.0f; if constexpr (TRAIN) op[mb][i] = 0.0f; }
    }
    float m = -INFINITY, lsum = 0.0f;     // lsum: this half-wave's part of l (same alpha in both halves)

    issue_tile(0, 0);
    // The Q registers must have arrived BEFORE the loop: a load still pending at loop entry makes the
    // compiler wait for all vector-memory traffic at the first product of every iteration, i.e. for
    // the tile prefetch it has just issued.
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) asm volatile("" : "+v"(qreg[ds]));
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int j = 0; j < nkt; ++j) {
        const int buf = j & 1;
        const int k0 = j * 64;
        if (j + 1 < nkt) issue_tile(buf ^ 1, j + 1);                    // lands while this tile is consumed
        const bool active = !CAUSAL || k0 <= wave_qmax;          // wave-uniform

        if (active) {
            // ---- S^T = K^F Q^F^T.  A wave sustains about one 1 KiB LDS read per 40 cycles and the
            // read latency is ~130 cycles, so the K operands are read RING steps ahead of the MFMA
            // that consumes them (the scheduling groups below keep the compiler from sinking them).
            floatx16 s[2];
            {
                // per-lane offset of this tile, opaque to the compiler: it would otherwise hoist every
                // (offset ^ constant) out of the loop and pay for it with registers
                int k_it = k_rd + buf * (int)sizeof(sm.k[0]);
                asm volatile("" : "+v"(k_it));
                const unsigned char* kbase = reinterpret_cast<const unsigned char*>(&sm.k[0][0]);
                auto k_opnd = [&](int i) __attribute__((always_inline)) -> half8 {
                    return __builtin_bit_cast(half8, lds_read16(kbase + (k_it ^ ((i >> 1) << 5)) + (i & 1) * (32 * D * 2)));
                };
                constexpr int NS = 2 * DS, RING = 6;
                half8 ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i)
                    ring[i] = k_opnd(i);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
#pragma unroll
                for (int i = 0; i < NS; ++i) {                  // step i: ds = i / 2, kb = i % 2
                    const half8 a = ring[i % RING];
                    if (i + RING < NS)
                        ring[i % RING] = k_opnd(i + RING);
                    s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[i >> 1], s[i & 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (i + RING < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            // ---- mask: keys beyond L, and keys after the query when causal
            const bool need_mask = (k0 + 64 > L) || (CAUSAL && k0 + 63 > qt * 128 + wave * 32);
            if (__builtin_expect(need_mask, 0)) {
                const int klim = CAUSAL ? min(L - 1, q_row) : L - 1;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = k0 + 32 * kb + 8 * (i >> 2) + 4 * hf + (i & 3);
                        if (key > klim) s[kb][i] = -INFINITY;
                    }
            }
            // ---- online softmax (Alg. 2: m_new, alpha, P-tilde, l)
            // (four interleaved chains each: a single chain of 32 dependent max / add instructions would
            // run at the instruction latency, not at the issue rate)
            float mp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) mp[j] = max_nc(s[0][j], s[1][j]);
#pragma unroll
            for (int i = 4; i < 16; ++i) mp[i & 3] = max_nc(max_nc(mp[i & 3], s[0][i]), s[1][i]);
            const float mt = xhalf_max(max_nc(max_nc(mp[0], mp[1]), max_nc(mp[2], mp[3])));
            const float mnew = fmaxf(m, mt);
            const float alpha = __builtin_amdgcn_exp2f((m - mnew) * c);
            const float ms = mnew * c;
            m = mnew;
            float rp[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -ms));
                    rp[i & 3] += s[kb][i];
                }
            const float rs = (rp[0] + rp[1]) + (rp[2] + rp[3]);
            lsum = lsum * alpha + rs;                           // un-quantized P-tilde
            // ---- rescale: exact no-op unless some row of this wave moved its maximum (rare
            // after the first tiles), so it lives on the cold path
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0, 0)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) { o[mb][i] *= alpha; if constexpr (TRAIN) op[mb][i] *= alpha; }
            }
            // ---- block scales of phi(P-tilde) for the four 16-key groups of the tile, as four independent
            // chains (max tree, exchange between the halves, E4M3 rounding, reciprocal): computed one after
            // the other they would sit on the critical path of every step below.
            float bsc[4], binv[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const floatx16& sv = s[ks >> 1];
                const int b0 = 8 * (ks & 1);
                const float a0 = fmaxf(fmaxf(sv[b0], sv[b0 + 1]), sv[b0 + 2]);
                const float a1 = fmaxf(fmaxf(sv[b0 + 3], sv[b0 + 4]), sv[b0 + 5]);
                bsc[ks] = fmaxf(fmaxf(a0, a1), fmaxf(sv[b0 + 6], sv[b0 + 7]));
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bsc[ks] = xhalf_max(bsc[ks]);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bsc[ks] = rne_e4m3_grid(bsc[ks] * (1.0f / 6.0f));   // P-tilde <= 1: no saturation
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) binv[ks] = bsc[ks] > 0.0f ? __builtin_amdgcn_rcpf(bsc[ks]) : 0.0f;
            // ---- per 16 keys: phi^-1(phi(P-tilde)), then O^T += V^F^T P-tilde^F^T and
            //      O'^T += V^F^T P-tilde^T.  Keys of a group = registers 8g..8g+7 of both halves.
            int v_it = v_rd + buf * (int)sizeof(sm.v[0]);
            asm volatile("" : "+v"(v_it));
            const unsigned char* vbase = reinterpret_cast<const unsigned char*>(&sm.v[0][0]);
            auto load_v = [&](int ks, half8 (&av)[MB]) __attribute__((always_inline)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    av[mb] = __builtin_bit_cast(half8, lds_read16(vbase + (v_it ^ (ks << 5)) + mb * (32 * 64 * 2)));
            };
            auto quantize = [&](int ks, uint4v& bq, uint4v& bu) __attribute__((always_inline)) {
                const int kb = ks >> 1, g = ks & 1;
                const float sc = bsc[ks], inv = binv[ks];
                const uint32_t sc2 = pack_f16x2(sc, sc);
                float pfv[DUMP ? 8 : 1];
                float r[8];
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = s[kb][8 * g + i] * inv;
                fq_oct_f16(r, sc2, w);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    bq[i] = w[i];
                    if constexpr (TRAIN) bu[i] = pack_f16x2(s[kb][8 * g + 2 * i], s[kb][8 * g + 2 * i + 1]);
                    if constexpr (DUMP) {
                        const half2v pr = __builtin_bit_cast(half2v, w[i]);
                        pfv[2 * i] = (float)pr[0]; pfv[2 * i + 1] = (float)pr[1];
                    }
                }
                if constexpr (DUMP) {
                    if (q_row >= dump_row0 && q_row < dump_row0 + 128 && q_row < L) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int key = k0 + 32 * kb + 16 * g + 8 * (i >> 2) + 4 * hf + (i & 3);
                            if (key < L)
                                pdump[((size_t)bh * 128 + (q_row - dump_row0)) * L + key] = pfv[i];
                        }
                    }
                }
            };
            if constexpr (DUMP) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    half8 av[MB];
                    uint4v bq, bu;
                    load_v(ks, av);
                    quantize(ks, bq, bu);
                    const half8 bqh = __builtin_bit_cast(half8, bq);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], bqh, o[mb], 0, 0, 0);
                        if constexpr (TRAIN)
                            op[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], __builtin_bit_cast(half8, bu), op[mb], 0, 0, 0);
                    }
                }
            } else {
                // A wave issues in order: a block of MFMAs followed by a block of vector instructions leaves
                // the vector ALU idle while the MFMAs queue up and the matrix pipe idle afterwards.  So the
                // quantization of step ks+1 is cut into four parts of a few instructions that follow the
                // products of step ks (scheduling fences keep the compiler from regrouping them); a V^T
                // operand register is reloaded for step ks+1 as soon as its last product of step ks has issued.
                struct QState { uint32_t c01, c23; };
                auto q_part = [&](int ks, int c, QState& st, uint4v& bq, uint4v& bu) __attribute__((always_inline)) {
                    const int b0 = 8 * (ks & 1);
                    const floatx16& sv = s[ks >> 1];
                    const float inv = binv[ks];
                    if (c == 0) {
                        st.c01 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, sv[b0] * inv, sv[b0 + 1] * inv, 1.0f, 0);
                        st.c23 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, sv[b0 + 4] * inv, sv[b0 + 5] * inv, 1.0f, 0);
                    } else if (c == 1) {
                        st.c01 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(st.c01, sv[b0 + 2] * inv, sv[b0 + 3] * inv, 1.0f, 1);
                        st.c23 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(st.c23, sv[b0 + 6] * inv, sv[b0 + 7] * inv, 1.0f, 1);
                    } else if (c == 2) {
                        const half2v sc2 = __builtin_bit_cast(half2v, pack_f16x2(bsc[ks], bsc[ks]));
                        bq[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c01, 1.0f, 0) * sc2);
                        bq[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c01, 1.0f, 1) * sc2);
                        bq[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c23, 1.0f, 0) * sc2);
                        bq[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(st.c23, 1.0f, 1) * sc2);
                    } else if constexpr (TRAIN) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) bu[i] = pack_f16x2(sv[b0 + 2 * i], sv[b0 + 2 * i + 1]);
                    }
                };
                half8 av[MB];
                uint4v bq[2], bu[2];
                QState st;
                load_v(0, av);
#pragma unroll
                for (int c = 0; c < 4; ++c) q_part(0, c, st, bq[0], bu[0]);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const int cur = ks & 1, nxt = cur ^ 1;
                    const half8 bqh = __builtin_bit_cast(half8, bq[cur]);
                    const half8 buh = __builtin_bit_cast(half8, bu[cur]);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        // the four parts of step ks+1 are spread over the MB operands of step ks
                        __builtin_amdgcn_sched_barrier(0);
                        o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], bqh, o[mb], 0, 0, 0);
                        if constexpr (TRAIN) {
                            __builtin_amdgcn_sched_barrier(0);
                            op[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], buh, op[mb], 0, 0, 0);
                        }
                        if (ks < 3) {
#pragma unroll
                            for (int c = (4 * mb) / MB; c < (4 * (mb + 1)) / MB; ++c) q_part(ks + 1, c, st, bq[nxt], bu[nxt]);
                        }
                        if (ks < 3) av[mb] = __builtin_bit_cast(half8, lds_read16(vbase + (v_it ^ ((ks + 1) << 5)) + mb * (32 * 64 * 2)));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);        // this wave's part of the next tile is in LDS
        __syncthreads();
    }

    // ---- epilogue: O /= l, O' /= l, L = m + log l
    const float l = xhalf_sum(lsum);
    const float inv_l = 1.0f / l;
    if (q_row < L) {
        const size_t row = (size_t)bh * L + q_row;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int d0 = 32 * mb + 8 * t + 4 * hf;
                uint2v w;
                w[0] = pack_bf16x2_rne(o[mb][4 * t] * inv_l, o[mb][4 * t + 1] * inv_l);
                w[1] = pack_bf16x2_rne(o[mb][4 * t + 2] * inv_l, o[mb][4 * t + 3] * inv_l);
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
}

template <int D, bool TRAIN, bool CAUSAL, bool DUMP>
static int launch_t(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int L,
                    void* o, float* lse, float* o_hp, int dump_row0, float* p_dump, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const int nqt = Lp / 128;
    const size_t smem = sizeof(FwdSmem<D>);
    auto kern = fwd_kernel<D, TRAIN, CAUSAL, DUMP>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)smem) != hipSuccess) return -1;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq * nqt)), dim3(256), smem, st,
                       (const half_t*)qh, (const half_t*)kh, (const half_t*)vt, (uint16_t*)o, lse, o_hp,
                       L, Lp, Hq, Hq / Hkv, c, dump_row0, p_dump);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D>
static int launch_d(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int L,
                    bool causal, bool train, void* o, float* lse, float* o_hp,
                    int dump_row0, float* p_dump, hipStream_t st)
{
    if (p_dump) {
        return causal ? launch_t<D, false, true, true>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, dump_row0, p_dump, st)
                      : launch_t<D, false, false, true>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, dump_row0, p_dump, st);
    }
    if (train) {
        return causal ? launch_t<D, true, true, false>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st)
                      : launch_t<D, true, false, false>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st);
    }
    return causal ? launch_t<D, false, true, false>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st)
                  : launch_t<D, false, false, false>(qh, kh, vt, B, Hq, Hkv, L, o, lse, o_hp, 0, nullptr, st);
}

int launch_fwd(const void* qh, const void* kh, const void* vt,
               int B, int Hq, int Hkv, int L, int D, bool causal, bool train,
               void* o, float* lse, float* o_hp, int dump_row0, float* p_dump, hipStream_t st)
{
    if (D == 128) return launch_d<128>(qh, kh, vt, B, Hq, Hkv, L, causal, train, o, lse, o_hp, dump_row0, p_dump, st);
    if (D == 64)  return launch_d<64>(qh, kh, vt, B, Hq, Hkv, L, causal, train, o, lse, o_hp, dump_row0, p_dump, st);
    return -1;
}

}  // namespace aq
