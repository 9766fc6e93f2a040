// Backward of Attn-QAT on gfx950 (Alg. 3), as four kernels:
//   delta      D = rowsum(dO o O') and the per-row {L, D} pairs   (first line of Alg. 3; HBM bound)
//   bounds     per-head maxima of |dO_i|, |V^F_j| and |D_i|: they bound |dS|   (HBM bound)
//   bwd_dq     query-stationary: S, P, dP, dS, dQ += dS K^F
//   bwd_dkdv   key-stationary:   S, P, P^F, dP, dS, dV += P^F^T dO, dK += dS^T Q^F
// The paper's single loop nest accumulates dQ across key tiles; here dQ gets its own pass
// that recomputes S and dP instead of accumulating across workgroups with atomics (the
// two-pass form of the Triton tutorial kernel the paper extends), which keeps every
// output deterministic.
//
// MFMA: v_mfma_f32_32x32x16_{f16,bf16}.  Q^F, K^F, V^F and P^F are exact in both 16-bit
// formats and dO is bf16 input, so S (fp16 operands), dP and dV (bf16 operands) see exact
// operands.  dS is fp32 and the only rounded operand: it enters its two products (with K^F
// and with Q^F, both fp16) as fp16, 11 significant bits, after multiplication by a power of
// two chosen from an upper bound of |dS| so that nothing overflows and the values that matter
// stay clear of the subnormals:
//     |dS_ij| = P_ij |dP_ij - D_i| / sqrt(d) <= (|dO_i| max_j |V^F_j| + |D_i|) / sqrt(d)
// (P <= 1, Cauchy-Schwarz).  The dQ pass scales per query row, the dK/dV pass per kv head; the
// accumulators are divided by the same power of two at the end.  A single bf16 (8 bits)
// would by itself cost about 1.7e-3 relative L2 in dQ and dK.
//
// As in the forward, S and dP are computed transposed ([key, query]) so that a lane owns
// one query row: L_i, D_i are per-lane scalars and the 16-key blocks of phi(P) are
// register reductions plus one exchange between the 32-lane halves.  Tiles are copied
// global->LDS directly (XOR-swizzled rows); operands that a product needs transposed
// (K^T for dQ; Q and dO column-wise, P^F^T and dS^T for dK/dV) are read from the row-major
// tiles with the LDS transpose read, so no transposed copy exists anywhere.
//
// LDS reads are the scarce resource of these loops (one wave sustains about one 1 KiB read
// per 40 cycles, latency ~130 cycles), so every operand read is issued a few MFMAs ahead of
// its consumer and the scheduling groups pin that order.
#include <type_traits>
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
__device__ inline floatx16 mfma_f16(uint4v a, uint4v b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}
// Largest power of two <= kDsTop / bound (bound >= 0), kept inside [2^-60, 2^60]: the factor that dS
// is multiplied by before it is rounded to fp16.
constexpr float kDsTop = 49152.0f;
__device__ inline float ds_scale_for(float bound) {
    float t = kDsTop / fmaxf(bound, 1e-30f);
    t = fminf(fmaxf(t, 8.7e-19f), 1.15e18f);
    return __uint_as_float(__float_as_uint(t) & 0x7F800000u);
}
__device__ inline uint4v join(uint2v a, uint2v b) { uint4v r; r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1]; return r; }

// ------------------------------------------------------------------ per-row statistics
// rowstat[bh*Lp + l] = { L_l * log2(e), D_l / sqrt(d) } with D = rowsum(dO o O'); rows l >= L
// (padding) hold {0, 0}.  Both attention passes read them as they are.
template <int D, bool LOWP /* ablation: O' is given as bf16 */>
__global__ __launch_bounds__(256) void delta_kernel(const uint16_t* __restrict__ dO, const void* __restrict__ Ohp_,
                                                    const float* __restrict__ lse,
                                                    int L, int Lp, long nrows_p, float rs, float2* __restrict__ rowstat)
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
        floatx4 o0, o1;
        if constexpr (LOWP) {
            const uint4v w = *reinterpret_cast<const uint4v*>(static_cast<const uint16_t*>(Ohp_) + off);
            o0[0] = bf16_lo_f32(w[0]); o0[1] = bf16_hi_f32(w[0]); o0[2] = bf16_lo_f32(w[1]); o0[3] = bf16_hi_f32(w[1]);
            o1[0] = bf16_lo_f32(w[2]); o1[1] = bf16_hi_f32(w[2]); o1[2] = bf16_lo_f32(w[3]); o1[3] = bf16_hi_f32(w[3]);
        } else {
            const float* Ohp = static_cast<const float*>(Ohp_);
            o0 = *reinterpret_cast<const floatx4*>(Ohp + off);
            o1 = *reinterpret_cast<const floatx4*>(Ohp + off + 4);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            acc += bf16_lo_f32(g[i]) * o0[2 * i] + bf16_hi_f32(g[i]) * o0[2 * i + 1];
            acc += bf16_lo_f32(g[2 + i]) * o1[2 * i] + bf16_hi_f32(g[2 + i]) * o1[2 * i + 1];
        }
    }
#pragma unroll
    for (int w = TPR / 2; w >= 1; w >>= 1) acc += __shfl_xor(acc, w);
    if (c == 0) rowstat[r] = make_float2(l < L ? lse[(size_t)bh * L + l] * 1.4426950408889634f : 0.0f, acc * rs);
}

int launch_delta(const void* d_o, const void* o_acc, bool o_is_bf16, const float* lse, int BHq, int L, int D,
                 float* rowstat, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const long nrows_p = (long)BHq * Lp;
    const int rpb = 256 / (D / 8);
    const unsigned grid = (unsigned)((nrows_p + rpb - 1) / rpb);
    const float rs = 1.0f / sqrtf((float)D);
    auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, (const uint16_t*)d_o, o_acc, lse, L, Lp, nrows_p, rs, (float2*)rowstat);
    };
    if (D == 128) { if (o_is_bf16) go(delta_kernel<128, true>); else go(delta_kernel<128, false>); }
    else          { if (o_is_bf16) go(delta_kernel<64, true>);  else go(delta_kernel<64, false>); }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ------------------------------------------------------------------ bounds of |dS|
// part[(which*NH + head)*kBoundParts + chunk]: maxima over the chunk's rows of
//   which 0: |V^F_j|_2 (kv heads)   1: |dO_i|_2 (query heads)   2: |D_i|/sqrt(d) (query heads)
// No atomics and no initialisation: the consumers reduce the kBoundParts partial maxima.
constexpr int kBoundParts = 64;

template <int D>
__global__ __launch_bounds__(256) void bounds_kernel(const uint16_t* __restrict__ Vb, const uint16_t* __restrict__ dOb,
                                                     const float2* __restrict__ rowstat, int Lp, int NHkv, int NHq,
                                                     float* __restrict__ part)
{
    constexpr int TPR = D / 8, RPP = 256 / TPR;      // threads per row, rows per pass
    __shared__ float red[2][4];
    const int head = blockIdx.x / kBoundParts, chunk = blockIdx.x % kBoundParts;      // 1-D grid: no 65535 limit on the heads
    const bool is_v = head < NHkv;
    const int h = is_v ? head : head - NHkv;
    const uint16_t* src = (is_v ? Vb : dOb) + (size_t)h * Lp * D;
    const int rows_per = (Lp + kBoundParts - 1) / kBoundParts;
    const int r_begin = chunk * rows_per, r_end = min(Lp, r_begin + rows_per);
    const int c = threadIdx.x % TPR;
    float nmax = 0.0f, dmax = 0.0f;
    for (int r = r_begin + threadIdx.x / TPR; r < r_end; r += RPP) {
        const uint4v g = *reinterpret_cast<const uint4v*>(src + (size_t)r * D + 8 * c);
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = bf16_lo_f32(g[i]), hi = bf16_hi_f32(g[i]);
            acc = fmaf(lo, lo, fmaf(hi, hi, acc));
        }
#pragma unroll
        for (int w = TPR / 2; w >= 1; w >>= 1) acc += __shfl_xor(acc, w);
        nmax = fmaxf(nmax, acc);
        if (!is_v && c == 0) dmax = fmaxf(dmax, fabsf(rowstat[(size_t)h * Lp + r].y));
    }
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) { nmax = fmaxf(nmax, __shfl_xor(nmax, w)); dmax = fmaxf(dmax, __shfl_xor(dmax, w)); }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = nmax; red[1][threadIdx.x >> 6] = dmax; }
    __syncthreads();
    if (threadIdx.x == 0) {
        nmax = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
        dmax = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
        const float nrm = sqrtf(nmax) * 1.0001f;     // rounded up a little: it is an upper bound
        if (is_v) part[(size_t)h * kBoundParts + chunk] = nrm;
        else {
            part[((size_t)NHq + h) * kBoundParts + chunk] = nrm;
            part[((size_t)2 * NHq + h) * kBoundParts + chunk] = dmax;
        }
    }
}

// One of the three maxima of a head: every lane gets the maximum of the head's partial values.
__device__ inline float bound_of(const float* __restrict__ part, int NHq, int which, int head) {
    float v = part[((size_t)which * NHq + head) * kBoundParts + (threadIdx.x & 63)];
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) v = fmaxf(v, __shfl_xor(v, w));
    return v;
}

int launch_bounds(const void* vb, const void* dob, const float* rowstat, int BHkv, int BHq, int L, int D,
                  float* part, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    dim3 grid((unsigned)kBoundParts * (unsigned)(BHkv + BHq));
    if (D == 128) hipLaunchKernelGGL(bounds_kernel<128>, grid, dim3(256), 0, st, (const uint16_t*)vb, (const uint16_t*)dob,
                                     (const float2*)rowstat, Lp, BHkv, BHq, part);
    else          hipLaunchKernelGGL(bounds_kernel<64>, grid, dim3(256), 0, st, (const uint16_t*)vb, (const uint16_t*)dob,
                                     (const float2*)rowstat, Lp, BHkv, BHq, part);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

static int g_bwd_waves = 0;           // waves per workgroup of the dQ and dK/dV passes, 0: chosen per problem; 4 / 8: forced (tests)
void set_bwd_waves(int waves) { __atomic_store_n(&g_bwd_waves, waves, __ATOMIC_RELAXED); }

// ------------------------------------------------------------------ dQ pass
template <int D, bool MXS>
struct DqSmem {
    uint16_t k[2][64 * D];       // K^F tile [key][d], fp16, swizzled
    uint16_t v[2][64 * D];       // V^F tile [key][d], bf16, swizzled
    unsigned char krec[MXS ? 2 : 1][MXS ? mx_ktrain_rec_bytes(D) : 16];      // MX: K operands of the FP4 instruction and their scales
};

typedef int int8v_t __attribute__((ext_vector_type(8)));
__device__ inline int8v_t fp4_opnd(const uint4v& x) {
    int8v_t r = {(int)x[0], (int)x[1], (int)x[2], (int)x[3], 0, 0, 0, 0};
    return r;
}

// MXS (the MX format): S^T = K^F Q^F^T is recomputed from the E2M1 codes and E8M0 scales by v_mfma_scale_f32_32x32x64_f8f6f4
// (Qops / Qsc: operands and scale dwords of the query rows, launch_mx_quant mode 1; Krec: the K records of mode 3); the
// accumulator layout is that of the 16-bit products, and dP, dS and dQ are computed as before (dO, dS are 16-bit values).
// NW waves of 32 query rows each share the K / V tiles: 4, or 8 for the passes of a large problem (half the
// tile copies per query row).
template <int D, bool CAUSAL, bool MXS, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void bwd_dq_kernel(
    const uint16_t* __restrict__ Qb, const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
    const uint16_t* __restrict__ dOb,
    const float2* __restrict__ rowstat, const float* __restrict__ bound_part, uint16_t* __restrict__ dQ,
    int L, int Lp, int Hq, int G, int NHq, float c /* log2e/sqrt(d) */, float rs /* 1/sqrt(d) */,
    const unsigned char* __restrict__ Qops, const uint32_t* __restrict__ Qsc, const unsigned char* __restrict__ Krec)
{
    constexpr int DS = D / 16, MB = D / 32, KCH = D / 8, KLD = KCH / NW, QT = 32 * NW /* query rows of a workgroup */;
    constexpr int KSM = D / 64, KREC = mx_ktrain_rec_bytes(D);
    extern __shared__ __align__(256) unsigned char smem_raw[];
    DqSmem<D, MXS>& sm = *reinterpret_cast<DqSmem<D, MXS>*>(smem_raw);

    const int nqt = (Lp + QT - 1) / QT;              // (Lp is a multiple of 128: with 8 waves the last workgroup may own only 128 rows)
    int bh, qt;
    head_tile_of_block(blockIdx.x, gridDim.x / nqt, nqt, bh, qt);
    if (CAUSAL) qt = nqt - 1 - qt;
    const int b = bh / Hq, h = bh % Hq;
    const int bhkv = b * (Hq / G) + h / G;
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // scalar: LDS destinations and branches use it
    const int q_row = qt * QT + wave * 32 + ln;
    const bool wave_live = NW == 4 || qt * QT + wave * 32 < Lp;      // a wave past the padded rows takes part in the copies and barriers only
    const int q_ld = wave_live ? q_row : ln;         // row its loads read instead

    uint4v qreg[MXS ? 1 : DS], doreg[DS], qop[MXS ? KSM : 1];
    uint32_t qs = 0u;
    {
        const size_t off = ((size_t)bh * Lp + q_ld) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            if constexpr (!MXS) qreg[ds] = *reinterpret_cast<const uint4v*>(Qb + off + 16 * ds);
            doreg[ds] = *reinterpret_cast<const uint4v*>(dOb + off + 16 * ds);
        }
        if constexpr (MXS) {
            const size_t grp = (size_t)bh * (Lp / 32) + ((q_ld - ln) >> 5);
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) qop[ks] = *reinterpret_cast<const uint4v*>(Qops + ((grp * KSM + ks) * 64 + lane) * 16);
            qs = Qsc[grp * 64 + lane];
        }
    }
    const float2 st_ = rowstat[(size_t)bh * Lp + q_ld];
    const float Ls = st_.x;                                          // L_i log2(e)
    // dS of this row goes to fp16 after multiplication by ds_scale = 2^k, k from the bound
    // (|dO_i| max_j |V^F_j| + |D_i|) / sqrt(d) >= |dS_ij|; rs_s and Dq_s carry the factor.
    float ds_scale;
    {
        float n2 = 0.0f;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float lo = bf16_lo_f32(doreg[ds][i]), hi = bf16_hi_f32(doreg[ds][i]);
                n2 = fmaf(lo, lo, fmaf(hi, hi, n2));
            }
        n2 = xhalf_sum(n2);
        const float vmax = bound_of(bound_part, NHq, 0, bhkv);
        ds_scale = ds_scale_for((sqrtf(n2) * 1.0001f * vmax) * rs + fabsf(st_.y));
    }
    const float rs_s = rs * ds_scale, Dq_s = st_.y * ds_scale;        // D_i / sqrt(d), scaled

    const int nkt_all = (L + 63) / 64;
    const int nkt = CAUSAL ? min((qt + 1) * (QT / 64), nkt_all) : nkt_all;
    const int wave_qmax = qt * QT + wave * 32 + 31;

    // direct-to-LDS tile loads: wave-uniform tile base + this lane's byte offset inside the tile
    uint32_t kv_ld[KLD];
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
        const int slot = 64 * (wave * KLD + i) + lane, r = slot / KCH, pc = slot % KCH;
        kv_ld[i] = 2u * (uint32_t)(r * D + 8 * swz<KCH>(r, pc));
    }
    const uint16_t* k_head = Kb + (size_t)bhkv * Lp * D;
    const uint16_t* v_head = Vb + (size_t)bhkv * Lp * D;
    const unsigned char* k_recs = MXS ? Krec + (size_t)bhkv * (Lp / 64) * KREC : nullptr;
    auto issue_tile = [&](int buf, int jt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < KLD; ++i) {
            async_copy16(k_head + (size_t)jt * (64 * D), kv_ld[i], &sm.k[buf][512 * (wave * KLD + i)]);
            async_copy16(v_head + (size_t)jt * (64 * D), kv_ld[i], &sm.v[buf][512 * (wave * KLD + i)]);
        }
        if constexpr (MXS) {
            for (int i = wave; i < KREC / 1024; i += NW)
                async_copy16(k_recs + (size_t)jt * KREC, (uint32_t)(i * 1024 + lane * 16), &sm.krec[buf][i * 1024]);
        }
    };

    // LDS element offsets (buffer 0).  Row blocks of 32 (kb) and key steps of 16 (ks) add
    // compile-time constants: they do not change a row's swizzle key.
    //   koff[ds]    16-byte operand reads of K and V rows: row ln, d-slots 16*ds + 8*hf
    //   toff[mb][v] transpose reads of K^T: lane r of a group of 16 points at key 4*hf + r/4 + 8*v,
    //               columns 32*mb + 16*grp + 4*(r%4); the lane receives column 32*mb + ln of 4 keys
    const int tr_r = lane & 15, tr_grp = (lane >> 4) & 1;
    // (LDS byte addresses inside buffer 0 of the K tile, as integers: with the buffer a compile-time constant in the loop
    //  below, every read is this register plus an immediate)
    const uint32_t k0_ad = lds_addr_of(&sm.k[0][0]);
    uint32_t koff[DS], toff[MB][2];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) koff[ds] = k0_ad + 2u * (uint32_t)((ln * KCH + swz<KCH>(ln, 2 * ds + hf)) * 8);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 2; ++v)
            toff[mb][v] = k0_ad + 2u * (uint32_t)swz_elem<KCH>(4 * hf + (tr_r >> 2) + 8 * v, 32 * mb + 16 * tr_grp + 4 * (tr_r & 3));
    constexpr uint32_t kTileB = 64 * D * 2, kVfromK = 2 * kTileB;      // bytes of a tile buffer; sm.v[b] lies kVfromK after sm.k[b]

    floatx16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;

    issue_tile(0, 0);
    // Q, dO and the row scalars must have arrived BEFORE the loop: a load still pending at loop entry
    // makes the compiler wait for all vector-memory traffic at the first product of every iteration,
    // i.e. for the tile prefetch it has just issued.
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
        if constexpr (!MXS) asm volatile("" : "+v"(qreg[ds]));
        asm volatile("" : "+v"(doreg[ds]));
    }
    if constexpr (MXS) {
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) asm volatile("" : "+v"(qop[ks]));
        asm volatile("" : "+v"(qs));
    }
    asm volatile("" :: "v"(Ls), "v"(rs_s), "v"(Dq_s));
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // one key tile; BUF = j mod 2 at compile time
    auto tile = [&](auto buf_tag, int j) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int k0 = j * 64;
        if (j + 1 < nkt) issue_tile(BUF ^ 1, j + 1);
        const bool active = (!CAUSAL || k0 <= wave_qmax) && wave_live;
        if (active) {
            floatx16 s[2], dp[2];
            if constexpr (MXS) {
                // S^T from the codes (2 * D/64 products), then dP^T = V^F dO^T: 2*DS steps, step i: ds = i/2, kb = i%2
                const uint32_t rec = lds_addr_of(&sm.krec[BUF][0]);
                const uint32_t ksc = *(const __attribute__((address_space(3))) uint32_t*)(uintptr_t)(rec + 2 * KSM * 1024 + lane * 4);
                uint4v a[2][KSM];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int ks = 0; ks < KSM; ++ks) a[kb][ks] = lds_read16_at(rec + (uint32_t)(((kb * KSM + ks) * 64 + lane) * 16));
                const floatx16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
                s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(a[0][0]), fp4_opnd(qop[0]), zero, 4, 4, 0, ksc, 0, qs);
                s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(a[1][0]), fp4_opnd(qop[0]), zero, 4, 4, KSM, ksc, 0, qs);
                if constexpr (KSM == 2) {
                    s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(a[0][1]), fp4_opnd(qop[1]), s[0], 4, 4, 1, ksc, 1, qs);
                    s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(a[1][1]), fp4_opnd(qop[1]), s[1], 4, 4, 3, ksc, 1, qs);
                }
                mfma_scale_settle(s[0], s[1]);
                constexpr int NST = 2 * DS, RING = 6;
                auto opnd = [&](int i) __attribute__((always_inline)) -> uint4v {
                    return lds_read16_at(koff[i >> 1] + (uint32_t)(BUF * kTileB + kVfromK + (i & 1) * (32 * D * 2)));
                };
                uint4v ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = opnd(i);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dp[kb][i] = 0.0f;
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    const uint4v av = ring[i % RING];
                    if (i + RING < NST) ring[i % RING] = opnd(i + RING);
                    dp[i & 1] = mfma_bf16(av, doreg[i >> 1], dp[i & 1]);
                }
            } else
            {   // S^T = K^F Q^F^T and dP^T = V^F dO^T: 4*DS steps, step i: ds = i/4, kb = (i/2)%2, K or V = i%2
                constexpr int NST = 4 * DS, RING = 6;
                auto opnd = [&](int i) __attribute__((always_inline)) -> uint4v {
                    return lds_read16_at(koff[i >> 2] + (uint32_t)(BUF * kTileB + (i & 1) * kVfromK + ((i >> 1) & 1) * (32 * D * 2)));
                };
                uint4v ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = opnd(i);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) { s[kb][i] = 0.0f; dp[kb][i] = 0.0f; }
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    const uint4v a = ring[i % RING];
                    if (i + RING < NST) ring[i % RING] = opnd(i + RING);
                    const int kb = (i >> 1) & 1, ds = i >> 2;
                    if (i & 1) dp[kb] = mfma_bf16(a, doreg[ds], dp[kb]);
                    else       s[kb] = mfma_f16(a, qreg[ds], s[kb]);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (i + RING < NST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            // masked keys (beyond L, or after the query): S = -inf so that P = 0
            const bool need_mask = (k0 + 64 > L) || (CAUSAL && k0 + 63 > qt * QT + wave * 32);
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
            // dQ^T += K^F^T dS^T, 16 keys per step; the K^T operands of a step are read (transposed)
            // before that step's dS is computed, so their latency hides behind the VALU work
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int kb = ks >> 1, g = ks & 1;
                uint4v at[MB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    at[mb] = join(lds_read_tr16_at(toff[mb][0] + (uint32_t)(BUF * kTileB + ks * (16 * D * 2))),
                                  lds_read_tr16_at(toff[mb][1] + (uint32_t)(BUF * kTileB + ks * (16 * D * 2))));
                uint4v bds;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r0 = 8 * g + 2 * i;
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][r0], c, -Ls));           // P = exp(S - L_i)
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][r0 + 1], c, -Ls));
                    // dS = P (dP - D_i)/sqrt(d), times ds_scale, to fp16
                    bds[i] = pack_f16x2(p0 * fmaf(dp[kb][r0], rs_s, -Dq_s), p1 * fmaf(dp[kb][r0 + 1], rs_s, -Dq_s));
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb] = mfma_f16(at[mb], bds, acc[mb]);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    for (int j = 0; j < nkt; j += 2) {
        tile(std::integral_constant<int, 0>{}, j);
        if (j + 1 < nkt) tile(std::integral_constant<int, 1>{}, j + 1);
    }

    if (q_row < L && wave_live) {
        const size_t row = (size_t)bh * L + q_row;
        const float un = rs / rs_s;                                  // 1 / ds_scale, exact: a power of two
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint2v w;
                w[0] = pack_bf16x2(acc[mb][4 * t] * un, acc[mb][4 * t + 1] * un);
                w[1] = pack_bf16x2(acc[mb][4 * t + 2] * un, acc[mb][4 * t + 3] * un);
                *reinterpret_cast<uint2v*>(dQ + row * D + 32 * mb + 8 * t + 4 * hf) = w;
            }
    }
}

template <int D, bool CAUSAL, bool MXS, int NW>
static int launch_dq_v(const void* qb, const void* kb, const void* vb, const void* dob,
                       const float* rowstat, const float* bound_part, int B, int Hq, int Hkv, int L, void* dq, hipStream_t st,
                       const MxScoreOps* mx)
{
    const int Lp = round_up(L, kRowPad);
    const size_t smem = sizeof(DqSmem<D, MXS>);
    auto kern = bwd_dq_kernel<D, CAUSAL, MXS, NW>;
    static unsigned long long lds_set = 0;          // one per instantiation
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return -1;
    const float rs = 1.0f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq * ((Lp + 32 * NW - 1) / (32 * NW)))), dim3(64 * NW), smem, st,
                       (const uint16_t*)qb, (const uint16_t*)kb, (const uint16_t*)vb,
                       (const uint16_t*)dob, (const float2*)rowstat, bound_part, (uint16_t*)dq, L, Lp, Hq, Hq / Hkv, B * Hq,
                       1.4426950408889634f * rs, rs,
                       (const unsigned char*)(mx ? mx->qops : nullptr), (const uint32_t*)(mx ? mx->qsc : nullptr),
                       (const unsigned char*)(mx ? mx->krec : nullptr));
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Eight waves per workgroup for a pass whose problem still leaves every compute unit two such workgroups to balance
// with, and, under a causal mask, whose sequences are long enough for the 256 rows at the diagonal, where part of the
// workgroup idles, not to matter (llm32k_gqa: 1.5 % faster with eight; llm4k_gqa: 2 - 8 % slower); or when a test
// forces them; four otherwise.
static bool wide_workgroups(bool causal, long long groups_of_256, int Lp)
{
    const int forced = __atomic_load_n(&g_bwd_waves, __ATOMIC_RELAXED);
    if (forced != 0) return forced == 8;
    return groups_of_256 >= 2LL * device_cu_count() && (!causal || Lp >= 16384);
}

template <int D, bool CAUSAL, bool MXS>
static int launch_dq_t(const void* qb, const void* kb, const void* vb, const void* dob,
                       const float* rowstat, const float* bound_part, int B, int Hq, int Hkv, int L, void* dq, hipStream_t st,
                       const MxScoreOps* mx)
{
    if (wide_workgroups(CAUSAL, (long long)B * Hq * ((round_up(L, kRowPad) + 255) / 256), round_up(L, kRowPad)))
        return launch_dq_v<D, CAUSAL, MXS, 8>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dq, st, mx);
    return launch_dq_v<D, CAUSAL, MXS, 4>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dq, st, mx);
}

int launch_bwd_dq(const void* qb, const void* kb, const void* vb, const void* dob,
                  const float* rowstat, const float* bound_part,
                  int B, int Hq, int Hkv, int L, int D, bool causal, void* dq, hipStream_t st, const MxScoreOps* mx)
{
    if (mx && (!mx->qops || !mx->qsc || !mx->krec)) return -1;
#define AQ_DQ(DD, C) (mx ? launch_dq_t<DD, C, true>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dq, st, mx) \
                         : launch_dq_t<DD, C, false>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dq, st, nullptr))
    if (D == 128) return causal ? AQ_DQ(128, true) : AQ_DQ(128, false);
    if (D == 64)  return causal ? AQ_DQ(64, true) : AQ_DQ(64, false);
#undef AQ_DQ
    return -1;
}

// ------------------------------------------------------------------ dK/dV pass
// A workgroup of NW waves owns 32 NW keys of one kv head (32 per wave, held in registers as MFMA A
// operands) and walks over the query rows of every query head of the group in tiles of 32.  NW = 4
// everywhere except the passes of a large problem (any format of P except the ablation), which run NW = 8: every
// Q / dO tile a workgroup fetches then serves twice the keys, which halves the pass's read traffic.
// The per-wave [query][key] staging tiles (32 queries x 32 keys, 16-bit values, rows of 64 bytes).  By the bank-conflict
// counter the LDS takes an 8-byte store from 16 lanes per cycle on 32 banks of 4 bytes and serves an 8-byte (transposing)
// read to 32 lanes per cycle on 64 banks.  A store instruction writes one 8-byte chunk of 16 consecutive queries per cycle,
// a read fetches the whole rows of four consecutive queries.  The rows of four consecutive queries (a group) are therefore
// contiguous, 256 bytes: a read touches every bank once.  For the stores every group is followed by 16 bytes of padding
// (the next group starts four banks further) and in the third and fourth row of a group neighbouring chunks are swapped:
// with the row's own 64 bytes = 16 banks that puts the 16 queries of a cycle on 16 different bank pairs.  (Rows padded
// to 72 bytes instead made every read collide once: 6 % of the pass's LDS cycles.)
constexpr int kTGroupB = 4 * 64 + 16;  // bytes of a group of four queries
constexpr int kTTileB = 8 * kTGroupB;  // bytes of a tile

template <int D, bool MXS, int NW>
struct DkvSmem {
    uint16_t q[2][32 * D];           // Q^F rows [query][d], fp16, swizzled
    uint16_t g[2][32 * D];           // dO rows  [query][d], bf16, swizzled
    uint16_t t[NW][2][kTTileB / 2];    // per wave: P^F (bf16) and dS (fp16, scaled) as [query][key]
    float rmax[NW][32];              // two-level P: per wave, the largest P of every query row over the wave's 32 keys
    unsigned char qrec[MXS ? 2 : 1][MXS ? (D / 64) * 1024 + 256 : 16];      // MX: Q operands of the FP4 instruction of a tile and their scale dwords
};

template <int D, bool CAUSAL, bool COUNT /* measurement / test variant: count tiles, dump P^F */,
          int PQ /* phi(P): 0 none (ablation: dV from the fp32 P), 1 NVFP4, 2 MX, 3 NVFP4 after the two-level row factor */,
          int NW = 4 /* waves, 32 keys each */>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void bwd_dkdv_kernel(
    const uint16_t* __restrict__ Qb, const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
    const uint16_t* __restrict__ dOb, const float2* __restrict__ rowstat, const float* __restrict__ bound_part,
    uint16_t* __restrict__ dK, uint16_t* __restrict__ dV, unsigned long long* __restrict__ tile_counts,
    int L, int Lp, int Hq, int G, int NHq, float c, float rs,
    float* __restrict__ pdump /* COUNT only, may be null: P^F of query rows [dump_row0, dump_row0 + 128), [B*Hq][128][L] */, int dump_row0,
    const unsigned char* __restrict__ Qops, const uint32_t* __restrict__ Qsc,      // PQ == 2 (MX) only: the scores come from the
    const unsigned char* __restrict__ Kops, const uint32_t* __restrict__ Ksc)      // codes, see bwd_dq_kernel
{
    constexpr bool MXS = PQ == 2;
    constexpr int KSM = D / 64, QREC = KSM * 1024 + 256;
    constexpr int DS = D / 16, NB = D / 32, KCH = D / 8;
    constexpr int NWL = (32 * KCH) / 64;             // 1 KiB wave-loads per tile of 32 rows
    constexpr int PER_WAVE = NWL >= NW ? NWL / NW : 1;
    extern __shared__ __align__(256) unsigned char smem_raw[];   // XORs of address bits 5..7 below commute with adding this base
    DkvSmem<D, MXS, NW>& sm = *reinterpret_cast<DkvSmem<D, MXS, NW>*>(smem_raw);

    constexpr int KT = 32 * NW;                      // keys of a workgroup
    const int nkt = (Lp + KT - 1) / KT;              // (Lp is a multiple of 128: with 8 waves the last workgroup may own only 128 keys)
    int bhkv, kt_;
    head_tile_of_block(blockIdx.x, gridDim.x / nkt, nkt, bhkv, kt_);    // key tiles in increasing order: under a causal
    const int Hkv = Hq / G;                         // mask the first tiles see the most queries
    const int b = bhkv / Hkv, hk = bhkv % Hkv;
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // scalar: LDS destinations and branches use it
    const int key0_w = kt_ * KT + wave * 32;        // this wave's first key
    const bool wave_live = NW == 4 || key0_w < Lp;  // a wave past the padded rows takes part in the copies and barriers only

    // K^F, V^F rows of this lane's key: A operands (row = key, d-slots 16*ds + 8*hf)
    uint4v kreg[MXS ? 1 : DS], vreg[DS], kop[MXS ? KSM : 1];
    uint32_t ksc = 0u;
    {
        const size_t off = ((size_t)bhkv * Lp + (wave_live ? key0_w : 0) + ln) * D + 8 * hf;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            if constexpr (!MXS) kreg[ds] = *reinterpret_cast<const uint4v*>(Kb + off + 16 * ds);
            vreg[ds] = *reinterpret_cast<const uint4v*>(Vb + off + 16 * ds);
        }
        if constexpr (MXS) {
            const size_t grp = (size_t)bhkv * (Lp / 32) + ((wave_live ? key0_w : 0) >> 5);
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) kop[ks] = *reinterpret_cast<const uint4v*>(Kops + ((grp * KSM + ks) * 64 + lane) * 16);
            ksc = Ksc[grp * 64 + lane];
        }
    }

    floatx16 dk[NB], dv[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[nb][i] = 0.0f; dv[nb][i] = 0.0f; }

    // query tiles of 32 rows, query heads of the group one after another; under a causal mask
    // only rows >= the workgroup's first key matter
    const int nq32 = (L + 31) / 32;
    const int qt_first = CAUSAL ? (kt_ * KT) / 32 : 0;
    const int per_head = nq32 - qt_first;
    const int niter = per_head > 0 ? per_head * G : 0;
    const size_t bh0 = (size_t)b * Hq + hk * G;      // first query head of the group

    // dS goes to fp16 after multiplication by ds_scale = 2^k, one k for the kv head, from the bound
    // (max_i |dO_i| max_j |V^F_j| + max_i |D_i|) / sqrt(d) >= |dS_ij| over the query heads of the group
    float ds_scale;
    {
        float domax = 0.0f, dmax = 0.0f;
        for (int g = 0; g < G; ++g) {
            domax = fmaxf(domax, bound_of(bound_part, NHq, 1, (int)bh0 + g));
            dmax = fmaxf(dmax, bound_of(bound_part, NHq, 2, (int)bh0 + g));
        }
        ds_scale = ds_scale_for(domax * bound_of(bound_part, NHq, 0, bhkv) * rs + dmax);
    }
    const float rs_s = rs * ds_scale;

    // direct-to-LDS loads: this wave's chunk slots and their (row, swizzled chunk)
    const bool loader = NWL >= NW || wave < NWL;
    uint32_t slot_off[PER_WAVE];                     // this lane's byte offset inside a tile's source rows
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int slot = 64 * (wave * PER_WAVE + i) + lane;
        slot_off[i] = 2u * (uint32_t)((slot / KCH) * D + 8 * swz<KCH>(slot / KCH, slot % KCH));
    }
    // (head, tile) walk without divisions: state of the NEXT tile to load and of the current tile
    int ld_g = 0, ld_t = 0;                          // next tile to issue: head index in group, tile in head
    auto issue_next = [&](int buf) __attribute__((always_inline)) {
        const size_t row0 = (bh0 + ld_g) * Lp + (size_t)(qt_first + ld_t) * 32;
        if (loader) {
#pragma unroll
            for (int i = 0; i < PER_WAVE; ++i) {
                async_copy16(Qb + row0 * D, slot_off[i], &sm.q[buf][512 * (wave * PER_WAVE + i)]);
                async_copy16(dOb + row0 * D, slot_off[i], &sm.g[buf][512 * (wave * PER_WAVE + i)]);
            }
        }
        if constexpr (MXS) {      // the tile's Q operands (KSM wave copies of 1 KiB) and their 64 scale dwords
            const size_t grp = (bh0 + ld_g) * (Lp / 32) + (size_t)(qt_first + ld_t);
            if (wave < KSM) async_copy16(Qops + grp * (KSM * 1024), (uint32_t)(wave * 1024 + lane * 16), &sm.qrec[buf][wave * 1024]);
            if (wave == 3 && lane < 16) async_copy16(Qsc + grp * 64, (uint32_t)(lane * 16), &sm.qrec[buf][KSM * 1024]);
        }
        if (++ld_t == per_head) { ld_t = 0; ++ld_g; }
    };

    // LDS byte offsets.  A row of a tile is D*2 bytes = KCH 16-byte chunks and chunk c of row r sits
    // at chunk c ^ key(r), so an offset is (per-lane constant) XOR (compile-time constant):
    //   operand reads of Q / dO rows (row ln, d-slots 16*ds + 8*hf):   a_rd ^ (ds << 5)
    //   transpose reads of Q / dO columns (lane r of a group of 16 points at query
    //   8*hf + r/4 + 4*v, columns 32*nb + 16*grp + 4*(r%4)):           g_rd[v] ^ (nb << 6)
    // 16 more rows, the other buffer and the dO tile are constant byte distances.
    constexpr int kRowB = 2 * D, kBufB = 32 * kRowB, kGB = 2 * kBufB;
    const int tr_r = lane & 15, tr_grp = (lane >> 4) & 1;
    const int a_rd = 2 * swz_elem<KCH>(ln, 8 * hf);
    int g_rd[2];
#pragma unroll
    for (int v = 0; v < 2; ++v) g_rd[v] = 2 * swz_elem<KCH>(8 * hf + (tr_r >> 2) + 4 * v, 16 * tr_grp + 4 * (tr_r & 3));
    // staging tiles of this wave, as LDS byte addresses (integers: pointer arithmetic on the dynamic LDS symbol costs an
    // add per access): this lane's writes and its transpose reads; the dS tile lies kTB bytes after the P^F tile
    constexpr int kTB = kTTileB;
    const uint32_t t_base = lds_addr_of(&sm.t[wave][0][0]);
    // writes: query ln, chunk hf + 2 t4 (keys 4 hf + 8 t4 .. + 3; t4 = 0..3 at compile time); reads: query 8 hf + tr_r/4 +
    // 16 ks + 4 s (group 2 hf + 4 ks + s), chunk 4 tr_grp + tr_r%4; the swap of neighbouring chunks flips the lane's part
    const uint32_t tw_ad = t_base + (uint32_t)(kTGroupB * (ln >> 2) + 64 * (ln & 3) + 8 * (hf ^ ((ln >> 1) & 1)));
    const uint32_t ta_ad = t_base + (uint32_t)(kTGroupB * (2 * hf) + 64 * (tr_r >> 2) + 32 * tr_grp + 8 * ((tr_r & 3) ^ ((tr_r >> 3) & 1)));
    const int lds0 = (int)lds_addr_of(smem_raw);

    // {L_i log2(e), D_i / sqrt(d)} of this lane's query row of the next tile
    float2 st_n = make_float2(0.0f, 0.0f);
    if (niter > 0) { issue_next(0); st_n = rowstat[bh0 * Lp + (size_t)qt_first * 32 + ln]; }
    // every load of the prologue must have arrived before the loop (see the dQ pass)
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
        if constexpr (!MXS) asm volatile("" : "+v"(kreg[ds]));
        asm volatile("" : "+v"(vreg[ds]));
    }
    if constexpr (MXS) {
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) asm volatile("" : "+v"(kop[ks]));
        asm volatile("" : "+v"(ksc));
    }
    asm volatile("" : "+v"(st_n.x), "+v"(st_n.y));
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    int cur_g = 0, cur_t = 0;
    unsigned n_tiles = 0, n_pf_tiles = 0;            // measurement only (wave-uniform)
    for (int it = 0; it < niter; ++it) {
        const int buf = it & 1;
        const int q0 = (qt_first + cur_t) * 32;
        const float Ls = st_n.x, Dq_s = st_n.y * (rs_s / rs);
        // next tile: start its copy and fetch its row scalars now, they are needed one iteration later
        int nx_g = cur_g, nx_t = cur_t + 1;
        if (nx_t == per_head) { nx_t = 0; ++nx_g; }
        if (it + 1 < niter) {
            issue_next(buf ^ 1);
            st_n = rowstat[(bh0 + nx_g) * Lp + (size_t)(qt_first + nx_t) * 32 + ln];
        }
        // wave-uniform.  With the two-level P every wave takes part in every tile: the exchange of the row maxima below
        // contains a workgroup barrier, and a wave whose keys all lie after the tile's queries computes P = 0 throughout
        // (which costs the first four query tiles of a workgroup some idle products and nothing else).
        const bool active = PQ == 3 || ((!CAUSAL || q0 + 31 >= key0_w) && wave_live);
        if (active) {
            // Q^F tile of this iteration (dO is kGB further).  The per-lane offsets are made opaque once
            // per iteration: otherwise the compiler hoists every (offset ^ constant) out of the loop and
            // pays for it with a dozen registers that this kernel does not have.
            int a_it = a_rd + buf * kBufB + lds0, g_it0 = g_rd[0] + buf * kBufB + lds0, g_it1 = g_rd[1] + buf * kBufB + lds0;
            asm volatile("" : "+v"(a_it), "+v"(g_it0), "+v"(g_it1));
            floatx16 s, dp;
            if constexpr (MXS) {
                // S^T from the codes (D/64 products), then dP^T = V^F dO^T over the dO tile (DS steps)
                const uint32_t rec = lds_addr_of(&sm.qrec[buf][0]);
                const uint32_t qsl = *(const __attribute__((address_space(3))) uint32_t*)(uintptr_t)(rec + KSM * 1024 + lane * 4);
                uint4v bq4[KSM];
#pragma unroll
                for (int ks = 0; ks < KSM; ++ks) bq4[ks] = lds_read16_at(rec + (uint32_t)((ks * 64 + lane) * 16));
                const floatx16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
                s = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(kop[0]), fp4_opnd(bq4[0]), zero, 4, 4, 0, ksc, 0, qsl);
                if constexpr (KSM == 2)
                    s = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_opnd(kop[1]), fp4_opnd(bq4[1]), s, 4, 4, 1, ksc, 1, qsl);
                mfma_scale_settle(s);
                constexpr int RING = 3;
                auto opnd = [&](int i) __attribute__((always_inline)) -> uint4v {
                    return lds_read16_at((uint32_t)((a_it ^ (i << 5)) + kGB));
                };
                uint4v ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = opnd(i);
#pragma unroll
                for (int i = 0; i < 16; ++i) dp[i] = 0.0f;
#pragma unroll
                for (int i = 0; i < DS; ++i) {
                    const uint4v bq = ring[i % RING];
                    if (i + RING < DS) ring[i % RING] = opnd(i + RING);
                    dp = mfma_bf16(vreg[i], bq, dp);
                }
            } else
            {   // S^T = K^F Q^F^T, dP^T = V^F dO^T: 2*DS steps, step i: ds = i/2, Q or dO = i%2
                // (the two-level variant carries the exchanged row maximum and its LDS slot on top: its ring is one shorter)
                constexpr int NST = 2 * DS, RING = PQ == 3 ? 2 : 3;
                auto opnd = [&](int i) __attribute__((always_inline)) -> uint4v {
                    return lds_read16_at((uint32_t)((a_it ^ ((i >> 1) << 5)) + (i & 1) * kGB));
                };
                uint4v ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = opnd(i);
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[i] = 0.0f; dp[i] = 0.0f; }
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    const uint4v bq = ring[i % RING];
                    if (i + RING < NST) ring[i % RING] = opnd(i + RING);
                    if (i & 1) dp = mfma_bf16(vreg[i >> 1], bq, dp);
                    else       s = mfma_f16(kreg[i >> 1], bq, s);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (i + RING < NST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            // masked keys (beyond L, or after the query): S = -inf so that P = 0
            const bool need_mask = (key0_w + 32 > L) || (CAUSAL && key0_w + 31 > q0);
            if (__builtin_expect(need_mask, 0)) {
                const int klim = CAUSAL ? min(L - 1, q0 + ln) : L - 1;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = key0_w + 8 * (i >> 2) + 4 * hf + (i & 3);
                    if (key > klim) s[i] = -INFINITY;
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c, -Ls));    // P = exp(S - L_i)
            // block scales of phi(P): one per 16 keys = registers 8*gq .. 8*gq+7 of both halves
            constexpr bool PQUANT = PQ != 0;
            float sc[2], inv[2];
            bool nz = false;
            if constexpr (PQ == 2) {
                // MX format: this wave's 32 keys are one block with a power-of-two scale
                float a4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) a4[t] = fmaxf(fmaxf(s[t], s[4 + t]), fmaxf(s[8 + t], s[12 + t]));
                const float amax = xhalf_max(fmaxf(fmaxf(a4[0], a4[1]), fmaxf(a4[2], a4[3])));
                const uint32_t byte = e8m0_of_amax(amax);
                sc[0] = sc[1] = e8m0_as_f32(byte);
                inv[0] = inv[1] = e8m0_inverse_as_f32(byte);
                nz = amax > 0.0f;
            } else if constexpr (PQ == 1) {
                // Is any block scale of this tile non-zero?  A scale is RNE_E4M3(amax / 6), which is zero exactly when
                // amax / 6 <= 2^-10 (half of the smallest subnormal, and the tie goes to the even neighbour, zero), and
                // it grows with amax: some block has a non-zero scale iff some lane's largest P passes that test.  The
                // scales themselves are only needed where the answer is yes (below).
                float p4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) p4[t] = fmaxf(fmaxf(s[t], s[4 + t]), fmaxf(s[8 + t], s[12 + t]));
                nz = fmaxf(fmaxf(p4[0], p4[1]), fmaxf(p4[2], p4[3])) * (1.0f / 6.0f) > 0.0009765625f;
            }
            // Two-level quantization of P (PQ == 3): the row factor belongs to an aligned group of 64 keys, the tile row
            // of the forward, i.e. to this wave's 32 keys and those of its neighbour (waves 0|1 and 2|3 of the
            // workgroup).  The two waves exchange their partial row maxima through LDS.
            float pair_max = 0.0f;
            if constexpr (PQ == 3) {
                float p4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) p4[t] = fmaxf(fmaxf(s[t], s[4 + t]), fmaxf(s[8 + t], s[12 + t]));
                const float own = xhalf_max(fmaxf(fmaxf(p4[0], p4[1]), fmaxf(p4[2], p4[3])));
                // rmax[w][row] sits 128 w + 4 row bytes into a 256-byte aligned array: the neighbour's slot is address ^ 128
                const uint32_t rm_ad = lds_addr_of(&sm.rmax[0][0]) + 128u * (uint32_t)wave + 4u * (uint32_t)ln;
                *(__attribute__((address_space(3))) float*)(uintptr_t)rm_ad = own;      // both half-waves hold the same value
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                pair_max = fmaxf(own, *(const __attribute__((address_space(3))) float*)(uintptr_t)(rm_ad ^ 128u));
            }
            // block scales of phi(P): one per 16 keys = registers 8*gq .. 8*gq+7 of both halves (NVFP4, with or without
            // the row factor of the two-level form)
            auto nvfp4_scales = [&]() __attribute__((always_inline)) {
                // Two-level quantization of P (PQ == 3): the row of the aligned 64-key group is divided by s1, the
                // smallest power of two with 2688 s1 >= max(row maximum of the group, 2^-24), before the NVFP4 blocks
                float s1 = 1.0f, inv1 = 1.0f;
                float amax[2];
#pragma unroll
                for (int gq = 0; gq < 2; ++gq) {
                    amax[gq] = s[8 * gq];
#pragma unroll
                    for (int i = 1; i < 8; ++i) amax[gq] = fmaxf(amax[gq], s[8 * gq + i]);
                    amax[gq] = xhalf_max(amax[gq]);
                }
                if constexpr (PQ == 3) {
                    const float base = fmaxf(pair_max, 5.9604644775390625e-08f);
                    const uint32_t e1 = ((__float_as_uint(base) + 0x0057FFFFu) >> 23) - 11u;      // 2688 = 1.3125 * 2^11
                    s1 = __uint_as_float(e1 << 23);
                    inv1 = __uint_as_float((254u - e1) << 23);
                }
                bool any = false;
#pragma unroll
                for (int gq = 0; gq < 2; ++gq) {
                    const float s2 = rne_e4m3_grid((amax[gq] * inv1) * (1.0f / 6.0f));
                    // P^F = (s1 s2) * code and the code is RNE(P / (s1 s2)): from here on the product of the two levels
                    // stands in for the block scale (a power of two times an E4M3 value: still exact in bf16)
                    sc[gq] = s2 * s1;
                    inv[gq] = s2 > 0.0f ? __builtin_amdgcn_rcpf(s2) * inv1 : 0.0f;
                    any = any || s2 > 0.0f;
                }
                return any;
            };
            if constexpr (PQ == 3) nz = nvfp4_scales();      // after the row factor a tile is almost never all zero
            // If every block scale of this 32x32 tile rounded to 0 (max P <= 6 * 2^-10: the usual case for long rows),
            // P^F is identically 0: quantizing it, staging it and the dV products are skipped.  Wave-uniform, exact.
            const bool with_pf = PQUANT && __builtin_amdgcn_ballot_w64(nz) != 0;
            if constexpr (COUNT) { ++n_tiles; if (with_pf) ++n_pf_tiles; }
            // P^F = phi^-1(phi(P)) as bf16, staged as [query][key] before dS is: both tiles are then in LDS when the
            // products start, and the dV products of a tile that has them follow its dK products in one stream (a wave
            // that quantized, staged and multiplied P^F only after its dK products kept the other three waiting at the
            // tile barrier for the whole of that dependent chain).
            if (with_pf) {
                if constexpr (PQ == 1) nvfp4_scales();
                if constexpr (PQUANT) {
#pragma unroll
                    for (int t4 = 0; t4 < 4; ++t4) {
                        const int r0 = 4 * t4, gq = t4 >> 1;
                        float pf[4];
                        fq_pair_f32(s[r0] * inv[gq], s[r0 + 1] * inv[gq], sc[gq], pf[0], pf[1]);
                        fq_pair_f32(s[r0 + 2] * inv[gq], s[r0 + 3] * inv[gq], sc[gq], pf[2], pf[3]);
                        uint2v wp;
                        wp[0] = pack_bf16x2(pf[0], pf[1]); wp[1] = pack_bf16x2(pf[2], pf[3]);
                        lds_write8_at(tw_ad + (uint32_t)(16 * t4), wp);
                        if constexpr (COUNT) {
                            const int qr = q0 + ln;      // registers r0 .. r0 + 3: keys key0_w + 8 t4 + 4 hf + e of query row qr
                            if (pdump && qr >= dump_row0 && qr < dump_row0 + 128 && qr < L) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const int key = key0_w + 8 * t4 + 4 * hf + e;
                                    if (key < L) pdump[((size_t)(bh0 + cur_g) * 128 + (qr - dump_row0)) * L + key] = pf[e];
                                }
                            }
                        }
                    }
                }
            }
            // dS = P (dP - D_i)/sqrt(d) from the fp32 P, scaled, as fp16, staged as [query][key]
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {                           // 4 consecutive keys per store
                const int r0 = 4 * t4;
                float dsv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) dsv[e] = s[r0 + e] * fmaf(dp[r0 + e], rs_s, -Dq_s);
                uint2v wh;
                wh[0] = pack_f16x2(dsv[0], dsv[1]); wh[1] = pack_f16x2(dsv[2], dsv[3]);
                // registers r0..r0+3 <-> keys 8*(r0>>2) + 4*hf + 0..3 of this wave's 32 keys
                lds_write8_at(tw_ad + (uint32_t)(kTB + 16 * t4), wh);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // dK += dS^T Q^F (steps 0 .. NSTEP-1) and dV += P^F^T dO (steps NSTEP .. 2 NSTEP-1), NSTEP = 2*NB steps each:
            // step j of a product covers queries 16*(j/NB) .. +15 (contraction slots 0-3: queries 16*ks + 8*hf + 0..3,
            // slots 4-7: the next four) and columns 32*(j%NB) .. +31.  The operands of a step are read while the step
            // before it multiplies.
            constexpr int NSTEP = 2 * NB;
            auto rd_b = [&](int j, int extra) __attribute__((always_inline)) -> uint4v {
                const int nb = j % NB, ks = j / NB;
                return join(lds_read_tr16_at((uint32_t)((g_it0 ^ (nb << 6)) + ks * (16 * kRowB) + extra)),
                            lds_read_tr16_at((uint32_t)((g_it1 ^ (nb << 6)) + ks * (16 * kRowB) + extra)));
            };
            auto rd_t = [&](int tb /* 0: P^F tile, kTB: dS tile */, int ks) __attribute__((always_inline)) -> uint4v {
                const uint32_t ta = ta_ad + (uint32_t)(tb + ks * (4 * kTGroupB));       // 16 rows = 4 groups further
                return join(lds_read_tr16_at(ta), lds_read_tr16_at(ta + kTGroupB));
            };
            // steps [FIRST, LAST) of the stream
            auto products = [&](auto first_tag, auto last_tag) __attribute__((always_inline)) {
                constexpr int FIRST = decltype(first_tag)::value, LAST = decltype(last_tag)::value;
                auto a_of = [&](int st) __attribute__((always_inline)) -> uint4v { return rd_t(st < NSTEP ? kTB : 0, (st % NSTEP) / NB); };
                auto b_of = [&](int st) __attribute__((always_inline)) -> uint4v { return rd_b(st % NSTEP, st < NSTEP ? 0 : kGB); };
                uint4v a = a_of(FIRST), b[2];
                b[FIRST & 1] = b_of(FIRST);
#pragma unroll
                for (int st = FIRST; st < LAST; ++st) {
                    const int nb = st % NB;
                    const bool new_a = st + 1 < LAST && (st + 1) % NB == 0;
                    if (st + 1 < LAST) b[(st + 1) & 1] = b_of(st + 1);
                    uint4v a_n;
                    if (new_a) a_n = a_of(st + 1);
                    if (st < NSTEP) dk[nb] = mfma_f16(a, b[st & 1], dk[nb]);
                    else            dv[nb] = mfma_bf16(a, b[st & 1], dv[nb]);
                    if (new_a) a = a_n;
                }
                __builtin_amdgcn_sched_group_barrier(0x100, 2 + 2, 0);
#pragma unroll
                for (int st = FIRST; st < LAST; ++st) {
                    if (st + 1 < LAST) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    if (st + 1 < LAST && (st + 1) % NB == 0) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
            };
            typedef std::integral_constant<int, 0> I0;
            typedef std::integral_constant<int, NSTEP> I1;
            typedef std::integral_constant<int, 2 * NSTEP> I2;
            if constexpr (PQUANT) {
                // (two branches, each with its whole stream, would let the dV operand reads start under the dK products; the
                //  compiler then shuffles the 256 accumulator registers between the branches and spills)
                products(I0{}, I1{});
                if (with_pf) products(I1{}, I2{});
            } else {
                // Ablation (Sec. 3.2, "no fake quantization of P in the backward"): dV from the fp32 P itself, which enters
                // its product in two passes as a bf16 hi + lo pair
                products(I0{}, I1{});
#pragma unroll
                for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                    for (int t4 = 0; t4 < 4; ++t4) {
                        const int r0 = 4 * t4;
                        float pf[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float hi = __uint_as_float((uint32_t)f32_to_bf16_rne(s[r0 + e]) << 16);
                            pf[e] = pass == 0 ? hi : s[r0 + e] - hi;
                        }
                        uint2v wp;
                        wp[0] = pack_bf16x2(pf[0], pf[1]); wp[1] = pack_bf16x2(pf[2], pf[3]);
                        lds_write8_at(tw_ad + (uint32_t)(16 * t4), wp);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    products(I1{}, I2{});
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        cur_g = nx_g; cur_t = nx_t;
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        asm volatile("" : "+v"(st_n.x), "+v"(st_n.y));     // the next tile's row scalars are consumed here, not earlier
    }

    if (COUNT && lane == 0 && tile_counts) {
        atomicAdd(&tile_counts[0], (unsigned long long)n_tiles);
        atomicAdd(&tile_counts[1], (unsigned long long)n_pf_tiles);
    }

    // accumulators: row = key 8*(i>>2) + 4*hf + (i&3) of the wave, column d = 32*nb + ln
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = key0_w + 8 * (i >> 2) + 4 * hf + (i & 3);
            if (key < L) {
                const size_t o = ((size_t)bhkv * L + key) * D + 32 * nb + ln;
                dK[o] = f32_to_bf16_rne(dk[nb][i] * (rs / rs_s));            // / ds_scale, exact: a power of two
                dV[o] = f32_to_bf16_rne(dv[nb][i]);
            }
        }
}

template <int D, bool CAUSAL, bool COUNT, int PQ, int NW>
static int launch_dkdv_v(const void* qb, const void* kb, const void* vb, const void* dob,
                         const float* rowstat, const float* bound_part,
                         int B, int Hq, int Hkv, int L, void* dk, void* dv, unsigned long long* tile_counts,
                         hipStream_t st, float* p_dump, int dump_row0, const MxScoreOps* mx)
{
    const int Lp = round_up(L, kRowPad);
    const size_t smem = sizeof(DkvSmem<D, PQ == 2, NW>);
    auto kern = bwd_dkdv_kernel<D, CAUSAL, COUNT, PQ, NW>;
    static unsigned long long lds_set = 0;          // one per instantiation
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return -1;
    const float rs = 1.0f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hkv * ((Lp + 32 * NW - 1) / (32 * NW)))), dim3(64 * NW), smem, st,
                       (const uint16_t*)qb, (const uint16_t*)kb, (const uint16_t*)vb,
                       (const uint16_t*)dob, (const float2*)rowstat, bound_part, (uint16_t*)dk, (uint16_t*)dv, tile_counts,
                       L, Lp, Hq, Hq / Hkv, B * Hq, 1.4426950408889634f * rs, rs, p_dump, dump_row0,
                       (const unsigned char*)(mx ? mx->qops : nullptr), (const uint32_t*)(mx ? mx->qsc : nullptr),
                       (const unsigned char*)(mx ? mx->kops : nullptr), (const uint32_t*)(mx ? mx->ksc : nullptr));
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D, bool CAUSAL>
static int launch_dkdv_t(const void* qb, const void* kb, const void* vb, const void* dob,
                         const float* rowstat, const float* bound_part,
                         int B, int Hq, int Hkv, int L, void* dk, void* dv, unsigned long long* tile_counts,
                         int p_quant, hipStream_t st, float* p_dump, int dump_row0, const MxScoreOps* mx)
{
    if (p_quant < 0 || p_quant > 3) return -1;
    if (p_quant == 2 && !(mx && mx->qops && mx->qsc && mx->kops && mx->ksc)) return -1;
    if (p_quant != 1) { if (p_dump) return -1; tile_counts = nullptr; }
#define AQ_DKV(COUNT, PQ, NW) launch_dkdv_v<D, CAUSAL, COUNT, PQ, NW>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dk, dv, \
                                                                       tile_counts, st, p_dump, dump_row0, mx)
    if (tile_counts || p_dump) return AQ_DKV(true, 1, 4);       // the counting / dumping variant
    if (p_quant == 0) return AQ_DKV(false, 0, 4);               // the ablation
    if (wide_workgroups(CAUSAL, (long long)B * Hkv * ((round_up(L, kRowPad) + 255) / 256), round_up(L, kRowPad)))
        return p_quant == 1 ? AQ_DKV(false, 1, 8) : p_quant == 2 ? AQ_DKV(false, 2, 8) : AQ_DKV(false, 3, 8);
    return p_quant == 1 ? AQ_DKV(false, 1, 4) : p_quant == 2 ? AQ_DKV(false, 2, 4) : AQ_DKV(false, 3, 4);
#undef AQ_DKV
}

int launch_bwd_dkdv(const void* qb, const void* kb, const void* vb, const void* dob,
                    const float* rowstat, const float* bound_part,
                    int B, int Hq, int Hkv, int L, int D, bool causal, void* dk, void* dv,
                    unsigned long long* tile_counts, int p_quant, hipStream_t st, float* p_dump, int dump_row0, const MxScoreOps* mx)
{
    if (D == 128) return causal ? launch_dkdv_t<128, true>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dk, dv, tile_counts, p_quant, st, p_dump, dump_row0, mx)
                                : launch_dkdv_t<128, false>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dk, dv, tile_counts, p_quant, st, p_dump, dump_row0, mx);
    if (D == 64)  return causal ? launch_dkdv_t<64, true>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dk, dv, tile_counts, p_quant, st, p_dump, dump_row0, mx)
                                : launch_dkdv_t<64, false>(qb, kb, vb, dob, rowstat, bound_part, B, Hq, Hkv, L, dk, dv, tile_counts, p_quant, st, p_dump, dump_row0, mx);
    return -1;
}

}  // namespace aq
