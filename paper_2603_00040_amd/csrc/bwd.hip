// Backward of Attn-QAT on gfx950 (Alg. 3), as three kernels:
//   delta      D = rowsum(dO o O')                        (first line of Alg. 3; HBM bound)
//   bwd_dq     query-stationary: S, P, dP, dS, dQ += dS K^F
//   bwd_dkdv   key-stationary:   S, P, P^F, dP, dS, dV += P^F^T dO, dK += dS^T Q^F
// The paper's single loop nest accumulates dQ across key tiles; here dQ gets its own pass
// that recomputes S and dP instead of accumulating across workgroups with atomics (the
// two-pass form of the Triton tutorial kernel the paper extends), which keeps every
// output deterministic.
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Q^F, K^F, V^F and P^F are exact in bf16 and dO is bf16
// input, so S, dP and dV see exact operands.  dS is fp32: it enters its two products as a
// bf16 pair hi + lo (hi = RNE(dS), lo = RNE(dS - hi)), which keeps 16 significant bits;
// a single bf16 would by itself cost about 1.7e-3 relative L2 in dQ and dK.
//
// As in the forward, S and dP are computed transposed ([key, query]) so that a lane owns
// one query row: L_i, D_i are per-lane scalars and the 16-key blocks of phi(P) are
// register reductions plus one exchange between the 32-lane halves.
#include "common.hpp"
#include "kernels.hpp"

namespace aq {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2 h; h[0] = (__bf16)lo; h[1] = (__bf16)hi;              // RNE
    return __builtin_bit_cast(uint32_t, h);
}
__device__ inline float bf16_lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline floatx16 mfma_bf16(uint4v a, uint4v b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------ delta
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const uint16_t* __restrict__ dO, const float* __restrict__ Ohp,
                                                    int L, int Lp, long nrows_p, float* __restrict__ delta)
{
    constexpr int TPR = D / 8;                 // threads per row
    const long r = (long)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;    // padded row id: bh*Lp + l
    const int c = threadIdx.x % TPR;
    if (r >= nrows_p) return;
    const long bh = r / Lp; const int l = (int)(r % Lp);
    float acc = 0.0f;
    if (l < L) {
        const size_t off = ((size_t)bh * L + l) * D + 8 * c;
        const uint4v g = *reinterpret_cast<const uint4v*>(dO + off);
        const floatx4 o0 = *reinterpret_cast<const floatx4*>(Ohp + off);
        const floatx4 o1 = *reinterpret_cast<const floatx4*>(Ohp + off + 4);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            acc += bf16_lo_f32(g[i]) * o0[2 * i] + bf16_hi_f32(g[i]) * o0[2 * i + 1];
            acc += bf16_lo_f32(g[2 + i]) * o1[2 * i] + bf16_hi_f32(g[2 + i]) * o1[2 * i + 1];
        }
    }
#pragma unroll
    for (int w = TPR / 2; w >= 1; w >>= 1) acc += __shfl_xor(acc, w);
    if (c == 0) delta[r] = acc;
}

int launch_delta(const void* d_o, const float* o_hp, int BHq, int L, int D, float* delta, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const long nrows_p = (long)BHq * Lp;
    const int rpb = 256 / (D / 8);
    const unsigned grid = (unsigned)((nrows_p + rpb - 1) / rpb);
    if (D == 128) hipLaunchKernelGGL(delta_kernel<128>, dim3(grid), dim3(256), 0, st, (const uint16_t*)d_o, o_hp, L, Lp, nrows_p, delta);
    else          hipLaunchKernelGGL(delta_kernel<64>, dim3(grid), dim3(256), 0, st, (const uint16_t*)d_o, o_hp, L, Lp, nrows_p, delta);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ------------------------------------------------------------------ dQ pass
template <int D>
struct DqSmem {
    uint16_t k[2][64][D + 8];       // K^F tile, row = key
    uint16_t v[2][64][D + 8];       // V^F tile, row = key
    uint16_t kt[2][D][64 + 8];      // K^F^T tile, row = d, keys permuted inside groups of 16
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void bwd_dq_kernel(
    const uint16_t* __restrict__ Qb, const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
    const uint16_t* __restrict__ Kt, const uint16_t* __restrict__ dOb,
    const float* __restrict__ lse, const float* __restrict__ delta, uint16_t* __restrict__ dQ,
    int L, int Lp, int Hq, int G, float c /* log2e/sqrt(d) */, float rs /* 1/sqrt(d) */)
{
    constexpr int DS = D / 16, MB = D / 32, KCH = D / 8, NLD = (64 * KCH) / 256;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    DqSmem<D>& sm = *reinterpret_cast<DqSmem<D>*>(smem_raw);

    const int nqt = Lp / 128;
    const int bh = blockIdx.x / nqt;
    int qt = blockIdx.x % nqt;
    if (CAUSAL) qt = nqt - 1 - qt;
    const int b = bh / Hq, h = bh % Hq;
    const int bhkv = b * (Hq / G) + h / G;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int q_row = qt * 128 + wave * 32 + ln;

    const uint16_t* Kbase = Kb + (size_t)bhkv * Lp * D;
    const uint16_t* Vbase = Vb + (size_t)bhkv * Lp * D;
    const uint16_t* Ktbase = Kt + (size_t)bhkv * D * Lp;

    uint4v qreg[DS], doreg[DS];
    {
        const size_t off = ((size_t)bh * Lp + q_row) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            qreg[ds] = *reinterpret_cast<const uint4v*>(Qb + off + 16 * ds);
            doreg[ds] = *reinterpret_cast<const uint4v*>(dOb + off + 16 * ds);
        }
    }
    const float Ls = (q_row < L ? lse[(size_t)bh * L + q_row] : 0.0f) * 1.4426950408889634f;
    const float Dq = delta[(size_t)bh * Lp + q_row];

    const int nkt_all = (L + 63) / 64;
    const int nkt = CAUSAL ? min(2 * qt + 2, nkt_all) : nkt_all;
    const int wave_qmax = qt * 128 + wave * 32 + 31;

    uint4v kld[NLD], vld[NLD], tld[NLD];
    auto gload = [&](int j) {
        const int k0 = j * 64;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            kld[i] = *reinterpret_cast<const uint4v*>(Kbase + (size_t)(k0 + ch / KCH) * D + 8 * (ch % KCH));
            vld[i] = *reinterpret_cast<const uint4v*>(Vbase + (size_t)(k0 + ch / KCH) * D + 8 * (ch % KCH));
            tld[i] = *reinterpret_cast<const uint4v*>(Ktbase + (size_t)(ch / 8) * Lp + k0 + 8 * (ch % 8));
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            *reinterpret_cast<uint4v*>(&sm.k[buf][ch / KCH][8 * (ch % KCH)]) = kld[i];
            *reinterpret_cast<uint4v*>(&sm.v[buf][ch / KCH][8 * (ch % KCH)]) = vld[i];
            *reinterpret_cast<uint4v*>(&sm.kt[buf][ch / 8][8 * (ch % 8)]) = tld[i];
        }
    };

    floatx16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;

    gload(0);
    sstore(0);
    __syncthreads();

    for (int j = 0; j < nkt; ++j) {
        const int buf = j & 1, k0 = j * 64;
        if (j + 1 < nkt) gload(j + 1);
        const bool active = !CAUSAL || k0 <= wave_qmax;
        uint32_t dsh[2][8], dsl[2][8];
        if (active) {
            floatx16 s[2], dp[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[kb][i] = 0.0f; dp[kb][i] = 0.0f; }
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) {
                    const uint4v ak = *reinterpret_cast<const uint4v*>(&sm.k[buf][32 * kb + ln][16 * ds + 8 * hf]);
                    s[kb] = mfma_bf16(ak, qreg[ds], s[kb]);                  // S^T = K^F Q^F^T
                    const uint4v av = *reinterpret_cast<const uint4v*>(&sm.v[buf][32 * kb + ln][16 * ds + 8 * hf]);
                    dp[kb] = mfma_bf16(av, doreg[ds], dp[kb]);              // dP^T = V^F dO^T
                }
            }
            const bool need_mask = (k0 + 64 > L) || (CAUSAL && k0 + 63 > qt * 128 + wave * 32);
            const int klim = CAUSAL ? min(L - 1, q_row) : L - 1;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float p = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -Ls));     // P = exp(S - L_i)
                    if (need_mask) {
                        const int key = k0 + 32 * kb + 8 * (i >> 2) + 4 * hf + (i & 3);
                        if (key > klim) p = 0.0f;
                    }
                    s[kb][i] = p * (dp[kb][i] - Dq) * rs;                          // dS, from the fp32 P
                }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t hi = pack_bf16x2(s[kb][2 * i], s[kb][2 * i + 1]);
                    dsh[kb][i] = hi;
                    dsl[kb][i] = pack_bf16x2(s[kb][2 * i] - bf16_lo_f32(hi), s[kb][2 * i + 1] - bf16_hi_f32(hi));
                }
        }
        if (j + 1 < nkt) sstore(buf ^ 1);
        if (active) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {                                       // dQ^T += K^F^T dS^T
                const int kb = ks >> 1, g = ks & 1;
                uint4v bh_, bl_;
#pragma unroll
                for (int i = 0; i < 4; ++i) { bh_[i] = dsh[kb][4 * g + i]; bl_[i] = dsl[kb][4 * g + i]; }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const uint4v a = *reinterpret_cast<const uint4v*>(&sm.kt[buf][32 * mb + ln][16 * ks + 8 * hf]);
                    acc[mb] = mfma_bf16(a, bh_, acc[mb]);
                    acc[mb] = mfma_bf16(a, bl_, acc[mb]);
                }
            }
        }
        __syncthreads();
    }

    if (q_row < L) {
        const size_t row = (size_t)bh * L + q_row;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint2v w;
                w[0] = pack_bf16x2(acc[mb][4 * t], acc[mb][4 * t + 1]);
                w[1] = pack_bf16x2(acc[mb][4 * t + 2], acc[mb][4 * t + 3]);
                *reinterpret_cast<uint2v*>(dQ + row * D + 32 * mb + 8 * t + 4 * hf) = w;
            }
    }
}

template <int D, bool CAUSAL>
static int launch_dq_t(const void* qb, const void* kb, const void* vb, const void* kt, const void* dob,
                       const float* lse, const float* delta, int B, int Hq, int Hkv, int L, void* dq, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const size_t smem = sizeof(DqSmem<D>);
    auto kern = bwd_dq_kernel<D, CAUSAL>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
        return -1;
    const float rs = 1.0f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq * (Lp / 128))), dim3(256), smem, st,
                       (const uint16_t*)qb, (const uint16_t*)kb, (const uint16_t*)vb, (const uint16_t*)kt,
                       (const uint16_t*)dob, lse, delta, (uint16_t*)dq, L, Lp, Hq, Hq / Hkv,
                       1.4426950408889634f * rs, rs);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_bwd_dq(const void* qb, const void* kb, const void* vb, const void* kt, const void* dob,
                  const float* lse, const float* delta,
                  int B, int Hq, int Hkv, int L, int D, bool causal, void* dq, hipStream_t st)
{
    if (D == 128) return causal ? launch_dq_t<128, true>(qb, kb, vb, kt, dob, lse, delta, B, Hq, Hkv, L, dq, st)
                                : launch_dq_t<128, false>(qb, kb, vb, kt, dob, lse, delta, B, Hq, Hkv, L, dq, st);
    if (D == 64)  return causal ? launch_dq_t<64, true>(qb, kb, vb, kt, dob, lse, delta, B, Hq, Hkv, L, dq, st)
                                : launch_dq_t<64, false>(qb, kb, vb, kt, dob, lse, delta, B, Hq, Hkv, L, dq, st);
    return -1;
}

// ------------------------------------------------------------------ dK/dV pass
// A workgroup owns 128 keys of one kv head (32 per wave, held in registers as MFMA A
// operands) and walks over the query rows of every query head of the group in tiles of 32.
template <int D>
struct DkvSmem {
    uint16_t q[2][32][D + 8];        // Q^F rows       (B operand of S^T)
    uint16_t g[2][32][D + 8];        // dO rows        (B operand of dP^T)
    uint16_t qt[2][D][32 + 8];       // Q^F^T          (B operand of dK), queries permuted in 16s
    uint16_t gt[2][D][32 + 8];       // dO^T           (B operand of dV)
    uint16_t t[4][3][32][32 + 8];    // per wave: P^F^T, dS_hi^T, dS_lo^T as [key][query] (A operands)
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void bwd_dkdv_kernel(
    const uint16_t* __restrict__ Qb, const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
    const uint16_t* __restrict__ Qt, const uint16_t* __restrict__ dOb, const uint16_t* __restrict__ dOt,
    const float* __restrict__ lse, const float* __restrict__ delta,
    uint16_t* __restrict__ dK, uint16_t* __restrict__ dV,
    int L, int Lp, int Hq, int G, float c, float rs)
{
    constexpr int DS = D / 16, NB = D / 32, KCH = D / 8;
    constexpr int NLD = (32 * KCH) / 256;            // 16-byte chunks per thread per tile
    extern __shared__ __align__(16) unsigned char smem_raw[];
    DkvSmem<D>& sm = *reinterpret_cast<DkvSmem<D>*>(smem_raw);

    const int nkt = Lp / 128;
    const int bhkv = blockIdx.x / nkt;
    const int kt_ = blockIdx.x % nkt;               // key tiles in increasing order: under a causal
    const int Hkv = Hq / G;                         // mask the first tiles see the most queries
    const int b = bhkv / Hkv, hk = bhkv % Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int key0_w = kt_ * 128 + wave * 32;       // this wave's first key
    const int key_row = key0_w + ln;

    // K^F, V^F rows of this lane's key: A operands (row = key, d-slots 16*ds + 8*hf)
    uint4v kreg[DS], vreg[DS];
    {
        const size_t off = ((size_t)bhkv * Lp + key_row) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            kreg[ds] = *reinterpret_cast<const uint4v*>(Kb + off + 16 * ds);
            vreg[ds] = *reinterpret_cast<const uint4v*>(Vb + off + 16 * ds);
        }
    }

    floatx16 dk[NB], dv[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[nb][i] = 0.0f; dv[nb][i] = 0.0f; }

    // query tiles of 32 rows; under a causal mask only rows >= the workgroup's first key matter
    const int nq32 = (L + 31) / 32;
    const int qt_first = CAUSAL ? (kt_ * 128) / 32 : 0;
    const int per_head = nq32 - qt_first;
    const int niter = per_head > 0 ? per_head * G : 0;

    uint4v ql[NLD], gl[NLD], qtl[NLD], gtl[NLD];
    auto gload = [&](int it) {
        const int g = it / per_head, q0 = (qt_first + it % per_head) * 32;
        const size_t bh = (size_t)b * Hq + hk * G + g;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            const size_t ro = (bh * Lp + q0 + ch / KCH) * D + 8 * (ch % KCH);
            ql[i] = *reinterpret_cast<const uint4v*>(Qb + ro);
            gl[i] = *reinterpret_cast<const uint4v*>(dOb + ro);
            const size_t to = (bh * D + ch / 4) * Lp + q0 + 8 * (ch % 4);
            qtl[i] = *reinterpret_cast<const uint4v*>(Qt + to);
            gtl[i] = *reinterpret_cast<const uint4v*>(dOt + to);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int ch = tid + 256 * i;
            *reinterpret_cast<uint4v*>(&sm.q[buf][ch / KCH][8 * (ch % KCH)]) = ql[i];
            *reinterpret_cast<uint4v*>(&sm.g[buf][ch / KCH][8 * (ch % KCH)]) = gl[i];
            *reinterpret_cast<uint4v*>(&sm.qt[buf][ch / 4][8 * (ch % 4)]) = qtl[i];
            *reinterpret_cast<uint4v*>(&sm.gt[buf][ch / 4][8 * (ch % 4)]) = gtl[i];
        }
    };

    if (niter > 0) { gload(0); sstore(0); }
    __syncthreads();

    // column of query ln inside a transposed tile: quads 1 and 2 of every 16 exchanged
    const int qcol = (ln & 16) | (ln & 3) | ((ln & 4) << 1) | ((ln & 8) >> 1);

    for (int it = 0; it < niter; ++it) {
        const int buf = it & 1;
        const int g = it / per_head, q0 = (qt_first + it % per_head) * 32;
        const size_t bh = (size_t)b * Hq + hk * G + g;
        if (it + 1 < niter) gload(it + 1);
        const bool active = !CAUSAL || q0 + 31 >= key0_w;          // wave-uniform
        if (active) {
            const int q_row = q0 + ln;
            const float Ls = (q_row < L ? lse[bh * L + q_row] : 0.0f) * 1.4426950408889634f;
            const float Dq = delta[bh * Lp + q_row];
            floatx16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.0f; dp[i] = 0.0f; }
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                const uint4v bq = *reinterpret_cast<const uint4v*>(&sm.q[buf][ln][16 * ds + 8 * hf]);
                s = mfma_bf16(kreg[ds], bq, s);                        // S^T = K^F Q^F^T
                const uint4v bg = *reinterpret_cast<const uint4v*>(&sm.g[buf][ln][16 * ds + 8 * hf]);
                dp = mfma_bf16(vreg[ds], bg, dp);                      // dP^T = V^F dO^T
            }
            // P = exp(S - L_i), masked keys (beyond L, or after the query) are 0
            const int klim = CAUSAL ? min(L - 1, q_row) : L - 1;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = key0_w + 8 * (i >> 2) + 4 * hf + (i & 3);
                const float p = __builtin_amdgcn_exp2f(fmaf(s[i], c, -Ls));
                s[i] = key > klim ? 0.0f : p;
            }
            uint16_t* tp = &sm.t[wave][0][0][0];
            uint16_t* th = &sm.t[wave][1][0][0];
            uint16_t* tl = &sm.t[wave][2][0][0];
#pragma unroll
            for (int gq = 0; gq < 2; ++gq) {                           // phi^-1(phi(P)) per 16 keys
                float amax = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, s[8 * gq + i]);
                amax = xhalf_max(amax);
                const float sc = rne_e4m3_grid(amax * (1.0f / 6.0f));
                const float inv = sc > 0.0f ? __builtin_amdgcn_rcpf(sc) : 0.0f;
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    const int r0 = 8 * gq + i;
                    const float pf0 = rne_e2m1_grid(fminf(s[r0] * inv, 6.0f)) * sc;
                    const float pf1 = rne_e2m1_grid(fminf(s[r0 + 1] * inv, 6.0f)) * sc;
                    const float ds0 = s[r0] * (dp[r0] - Dq) * rs;       // dS from the fp32 P
                    const float ds1 = s[r0 + 1] * (dp[r0 + 1] - Dq) * rs;
                    const uint32_t wp = pack_bf16x2(pf0, pf1);
                    const uint32_t wh = pack_bf16x2(ds0, ds1);
                    const uint32_t wl = pack_bf16x2(ds0 - bf16_lo_f32(wh), ds1 - bf16_hi_f32(wh));
                    // register r <-> key row 8*(r>>2) + 4*hf + (r&3) of this wave's 32 keys
                    const int kr0 = 8 * (r0 >> 2) + 4 * hf + (r0 & 3);
                    const int o0 = kr0 * 40 + qcol, o1 = o0 + 40;
                    tp[o0] = (uint16_t)wp; tp[o1] = (uint16_t)(wp >> 16);
                    th[o0] = (uint16_t)wh; th[o1] = (uint16_t)(wh >> 16);
                    tl[o0] = (uint16_t)wl; tl[o1] = (uint16_t)(wl >> 16);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {                           // 16 queries per step
                const uint4v ap = *reinterpret_cast<const uint4v*>(&sm.t[wave][0][ln][16 * ks + 8 * hf]);
                const uint4v ah = *reinterpret_cast<const uint4v*>(&sm.t[wave][1][ln][16 * ks + 8 * hf]);
                const uint4v al = *reinterpret_cast<const uint4v*>(&sm.t[wave][2][ln][16 * ks + 8 * hf]);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const uint4v bg = *reinterpret_cast<const uint4v*>(&sm.gt[buf][32 * nb + ln][16 * ks + 8 * hf]);
                    dv[nb] = mfma_bf16(ap, bg, dv[nb]);                // dV += P^F^T dO
                    const uint4v bq = *reinterpret_cast<const uint4v*>(&sm.qt[buf][32 * nb + ln][16 * ks + 8 * hf]);
                    dk[nb] = mfma_bf16(ah, bq, dk[nb]);                // dK += dS^T Q^F
                    dk[nb] = mfma_bf16(al, bq, dk[nb]);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (it + 1 < niter) sstore(buf ^ 1);
        __syncthreads();
    }

    // accumulators: row = key 8*(i>>2) + 4*hf + (i&3) of the wave, column d = 32*nb + ln
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = key0_w + 8 * (i >> 2) + 4 * hf + (i & 3);
            if (key < L) {
                const size_t o = ((size_t)bhkv * L + key) * D + 32 * nb + ln;
                dK[o] = f32_to_bf16_rne(dk[nb][i]);
                dV[o] = f32_to_bf16_rne(dv[nb][i]);
            }
        }
}

template <int D, bool CAUSAL>
static int launch_dkdv_t(const void* qb, const void* kb, const void* vb, const void* qt, const void* dob,
                         const void* dot, const float* lse, const float* delta,
                         int B, int Hq, int Hkv, int L, void* dk, void* dv, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const size_t smem = sizeof(DkvSmem<D>);
    auto kern = bwd_dkdv_kernel<D, CAUSAL>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
        return -1;
    const float rs = 1.0f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hkv * (Lp / 128))), dim3(256), smem, st,
                       (const uint16_t*)qb, (const uint16_t*)kb, (const uint16_t*)vb, (const uint16_t*)qt,
                       (const uint16_t*)dob, (const uint16_t*)dot, lse, delta, (uint16_t*)dk, (uint16_t*)dv,
                       L, Lp, Hq, Hq / Hkv, 1.4426950408889634f * rs, rs);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_bwd_dkdv(const void* qb, const void* kb, const void* vb, const void* qt, const void* dob,
                    const void* dot, const float* lse, const float* delta,
                    int B, int Hq, int Hkv, int L, int D, bool causal, void* dk, void* dv, hipStream_t st)
{
    if (D == 128) return causal ? launch_dkdv_t<128, true>(qb, kb, vb, qt, dob, dot, lse, delta, B, Hq, Hkv, L, dk, dv, st)
                                : launch_dkdv_t<128, false>(qb, kb, vb, qt, dob, dot, lse, delta, B, Hq, Hkv, L, dk, dv, st);
    if (D == 64)  return causal ? launch_dkdv_t<64, true>(qb, kb, vb, qt, dob, dot, lse, delta, B, Hq, Hkv, L, dk, dv, st)
                                : launch_dkdv_t<64, false>(qb, kb, vb, qt, dob, dot, lse, delta, B, Hq, Hkv, L, dk, dv, st);
    return -1;
}

}  // namespace aq
