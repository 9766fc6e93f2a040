// Fused forward of Attn-QAT on gfx950: Alg. 1 (inference) and Alg. 2 (training).
//
// Work split: a workgroup of 4 waves owns 128 query rows of one head; each wave owns 32
// of them.  Key tiles of B_k = 64 keys are visited in increasing order; K and V^T tiles
// are staged through LDS (double buffered) and shared by the four waves.
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
    half_t k[2][64][D + 8];      // K tile, row = key; +16 B pad: conflict-free 16 B reads
    half_t v[2][D][64 + 8];      // V^T tile, row = d
};

template <int D, bool TRAIN, bool CAUSAL, bool DUMP>
__global__ __launch_bounds__(256) void fwd_kernel(
    const half_t* __restrict__ Qh, const half_t* __restrict__ Kh, const half_t* __restrict__ Vt,
    uint16_t* __restrict__ O, float* __restrict__ lse, float* __restrict__ Ohp,
    int L, int Lp, int Hq, int G, float c /* log2(e)/sqrt(d) */, int dump_row0, float* __restrict__ pdump)
{
    constexpr int DS = D / 16;      // contraction steps of S
    constexpr int MB = D / 32;      // 32-row blocks of O^T
    constexpr int KCH = D / 8;      // 16-byte chunks per K row
    constexpr int NLD = (64 * KCH) / 256;   // chunks per thread per tile (K and V^T alike)
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

    const half_t* Kbase = Kh + (size_t)bhkv * Lp * D;
    const half_t* Vbase = Vt + (size_t)bhkv * D * Lp;

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

    uint4v kld[NLD], vld[NLD];
    auto gload = [&](int j) {
        const int k0 = j * 64;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            kld[i] = *reinterpret_cast<const uint4v*>(Kbase + (size_t)(k0 + ch / KCH) * D + 8 * (ch % KCH));
            vld[i] = *reinterpret_cast<const uint4v*>(Vbase + (size_t)(ch / 8) * Lp + k0 + 8 * (ch % 8));
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            *reinterpret_cast<uint4v*>(&sm.k[buf][ch / KCH][8 * (ch % KCH)]) = kld[i];
            *reinterpret_cast<uint4v*>(&sm.v[buf][ch / 8][8 * (ch % 8)]) = vld[i];
        }
    };

    floatx16 o[MB], op[TRAIN ? MB : 1];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { o[mb][i] = 0.0f; if constexpr (TRAIN) op[mb][i] = 0.0f; }
    }
    float m = -INFINITY, lsum = 0.0f;     // lsum: this half-wave's part of l (same alpha in both halves)

    gload(0);
    sstore(0);
    __syncthreads();

    for (int j = 0; j < nkt; ++j) {
        const int buf = j & 1;
        const int k0 = j * 64;
        if (j + 1 < nkt) gload(j + 1);
        const bool active = !CAUSAL || k0 <= wave_qmax;          // wave-uniform

        floatx16 s[2];
        uint32_t pq[2][8], pu[TRAIN ? 2 : 1][8];                 // packed fp16 P-tilde^F / P-tilde
        float alpha = 1.0f;
        if (active) {
            // ---- S^T = K^F Q^F^T
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) {
                    const half8 a = *reinterpret_cast<const half8*>(&sm.k[buf][32 * kb + ln][16 * ds + 8 * hf]);
                    s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qreg[ds], s[kb], 0, 0, 0);
                }
            }
            // ---- mask: keys beyond L, and keys after the query when causal
            const bool need_mask = (k0 + 64 > L) || (CAUSAL && k0 + 63 > qt * 128 + wave * 32);
            if (need_mask) {
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
            float mt = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s[kb][i]);
            mt = xhalf_max(mt);
            const float mnew = fmaxf(m, mt);
            alpha = __builtin_amdgcn_exp2f((m - mnew) * c);
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
            // ---- phi^-1(phi(P-tilde)): groups of 16 keys = registers 8g..8g+7 of both halves
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    float amax = 0.0f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, s[kb][8 * g + i]);
                    amax = xhalf_max(amax);
                    const float sc = rne_e4m3_grid(amax * (1.0f / 6.0f));   // P-tilde <= 1: no saturation
                    const float inv = sc > 0.0f ? __builtin_amdgcn_rcpf(sc) : 0.0f;
                    float pf[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        pf[i] = rne_e2m1_grid(fminf(s[kb][8 * g + i] * inv, 6.0f)) * sc;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        pq[kb][4 * g + i] = pack_f16x2(pf[2 * i], pf[2 * i + 1]);
                        if constexpr (TRAIN) pu[kb][4 * g + i] = pack_f16x2(s[kb][8 * g + 2 * i], s[kb][8 * g + 2 * i + 1]);
                    }
                    if constexpr (DUMP) {
                        if (q_row >= dump_row0 && q_row < dump_row0 + 128 && q_row < L) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const int key = k0 + 32 * kb + 16 * g + 8 * (i >> 2) + 4 * hf + (i & 3);
                                if (key < L)
                                    pdump[((size_t)bh * 128 + (q_row - dump_row0)) * L + key] = pf[i];
                            }
                        }
                    }
                }
        }
        // stage the next tile while this one is still being consumed
        if (j + 1 < nkt) sstore(buf ^ 1);

        if (active) {
            // ---- rescale, exact no-op when no row of this wave moved its maximum
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) { o[mb][i] *= alpha; if constexpr (TRAIN) op[mb][i] *= alpha; }
            }
            // ---- O^T += V^F^T P-tilde^F^T ; O'^T += V^F^T P-tilde^T
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int kb = ks >> 1, g = ks & 1;
                uint4v bq; bq[0] = pq[kb][4 * g]; bq[1] = pq[kb][4 * g + 1]; bq[2] = pq[kb][4 * g + 2]; bq[3] = pq[kb][4 * g + 3];
                const half8 bqh = __builtin_bit_cast(half8, bq);
                half8 buh;
                if constexpr (TRAIN) {
                    uint4v bu; bu[0] = pu[kb][4 * g]; bu[1] = pu[kb][4 * g + 1]; bu[2] = pu[kb][4 * g + 2]; bu[3] = pu[kb][4 * g + 3];
                    buh = __builtin_bit_cast(half8, bu);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const half8 a = *reinterpret_cast<const half8*>(&sm.v[buf][32 * mb + ln][16 * ks + 8 * hf]);
                    o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bqh, o[mb], 0, 0, 0);
                    if constexpr (TRAIN) op[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, buh, op[mb], 0, 0, 0);
                }
            }
        }
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
