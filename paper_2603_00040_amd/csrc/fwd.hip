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
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
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
    int koff[DS], voff[4];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) koff[ds] = (ln * KCH + swz<KCH>(ln, 2 * ds + hf)) * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) voff[ks] = (ln * 8 + swz<8>(ln, 2 * ks + hf)) * 8;

    // per-lane global sources of the direct-to-LDS tile loads (advance by one tile per step)
    const half_t* ksrc[KLD];
    const half_t* vsrc[VLD];
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
        const int slot = 64 * (wave * KLD + i) + lane, r = slot / KCH, pc = slot % KCH;
        ksrc[i] = Kh + ((size_t)bhkv * Lp + r) * D + 8 * swz<KCH>(r, pc);
    }
#pragma unroll
    for (int i = 0; i < VLD; ++i) {
        const int slot = 64 * (wave * VLD + i) + lane, r = slot / 8, pc = slot % 8;
        vsrc[i] = Vt + ((size_t)bhkv * D + r) * Lp + 8 * swz<8>(r, pc);
    }
    auto issue_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < KLD; ++i) { async_copy16(ksrc[i], &sm.k[buf][512 * (wave * KLD + i)]); ksrc[i] += 64 * D; }
#pragma unroll
        for (int i = 0; i < VLD; ++i) { async_copy16(vsrc[i], &sm.v[buf][512 * (wave * VLD + i)]); vsrc[i] += 64; }
    };

    floatx16 o[MB], op[TRAIN ? MB : 1];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { o[mb][i] = 0.0f; if constexpr (TRAIN) op[mb][i] = 0.0f; }
    }
    float m = -INFINITY, lsum = 0.0f;     // lsum: this half-wave's part of l (same alpha in both halves)

    issue_tile(0);
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
        if (j + 1 < nkt) issue_tile(buf ^ 1);                    // lands while this tile is consumed
        const bool active = !CAUSAL || k0 <= wave_qmax;          // wave-uniform

        if (active) {
            // ---- S^T = K^F Q^F^T.  A wave sustains about one 1 KiB LDS read per 40 cycles and the
            // read latency is ~130 cycles, so the K operands are read RING steps ahead of the MFMA
            // that consumes them (the scheduling groups below keep the compiler from sinking them).
            floatx16 s[2];
            {
                const half_t* kt_ = &sm.k[buf][0];
                constexpr int NS = 2 * DS, RING = 6;
                half8 ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i)
                    ring[i] = *reinterpret_cast<const half8*>(kt_ + koff[i >> 1] + (i & 1) * (32 * D));
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
#pragma unroll
                for (int i = 0; i < NS; ++i) {                  // step i: ds = i / 2, kb = i % 2
                    const half8 a = ring[i % RING];
                    if (i + RING < NS)
                        ring[i % RING] = *reinterpret_cast<const half8*>(kt_ + koff[(i + RING) >> 1] + ((i + RING) & 1) * (32 * D));
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
            float mt = fmaxf(s[0][0], s[1][0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) mt = fmaxf(mt, fmaxf(s[0][i], s[1][i]));
            mt = xhalf_max(mt);
            const float mnew = fmaxf(m, mt);
            const float alpha = __builtin_amdgcn_exp2f((m - mnew) * c);
            const float ms = mnew * c;
            m = mnew;
            float rs = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -ms));
                    rs += s[kb][i];
                }
            lsum = lsum * alpha + rs;                           // un-quantized P-tilde
            // ---- rescale: exact no-op unless some row of this wave moved its maximum (rare
            // after the first tiles), so it lives on the cold path
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0, 0)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) { o[mb][i] *= alpha; if constexpr (TRAIN) op[mb][i] *= alpha; }
            }
            // ---- per 16 keys: phi^-1(phi(P-tilde)), then O^T += V^F^T P-tilde^F^T and
            //      O'^T += V^F^T P-tilde^T.  Keys of a group = registers 8g..8g+7 of both halves.
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int kb = ks >> 1, g = ks & 1;
                half8 av[MB];                                   // this step's V^F^T operands, in flight during phi
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    av[mb] = *reinterpret_cast<const half8*>(&sm.v[buf][voff[ks] + mb * (32 * 64)]);
                float amax = s[kb][8 * g];
#pragma unroll
                for (int i = 1; i < 8; ++i) amax = fmaxf(amax, s[kb][8 * g + i]);
                amax = xhalf_max(amax);
                const float sc = rne_e4m3_grid(amax * (1.0f / 6.0f));   // P-tilde <= 1: no saturation
                const float inv = sc > 0.0f ? __builtin_amdgcn_rcpf(sc) : 0.0f;
                const uint32_t sc2 = pack_f16x2(sc, sc);
                uint4v bq, bu;
                float pfv[DUMP ? 8 : 1];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p0 = s[kb][8 * g + 2 * i], p1 = s[kb][8 * g + 2 * i + 1];
                    const uint32_t w = fq_pair_f16(p0 * inv, p1 * inv, sc2);
                    bq[i] = w;
                    if constexpr (TRAIN) bu[i] = pack_f16x2(p0, p1);
                    if constexpr (DUMP) {
                        const half2v pr = __builtin_bit_cast(half2v, w);
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
                const half8 bqh = __builtin_bit_cast(half8, bq);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], bqh, o[mb], 0, 0, 0);
                    if constexpr (TRAIN)
                        op[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[mb], __builtin_bit_cast(half8, bu), op[mb], 0, 0, 0);
                }
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
