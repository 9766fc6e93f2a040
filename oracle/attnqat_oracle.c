/*
 * CPU oracle for NVFP4 fake-quantized attention (Attn-QAT).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, and meant to be checked against the
 * paper by eye.  It shares no code with the HIP library and is used only by
 * the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Arithmetic: fp64 everywhere, except that the operand of every phi(P) is
 * first rounded to fp32 (the softmax is an fp32 quantity in the method,
 * Sec. 2.3 "High-precision O for the backward pass"), and phi's rounding
 * decisions are taken exactly on those fp32 values.
 *
 * What is implemented
 *   phi / phi^-1           Sec. 2.1 "NVFP4 and SageAttention3", Eq. 1 and Eq. 2
 *   forward (train+infer)  Alg. 2 "Attn-QAT Forward (Training)"; Alg. 1 is the
 *                          same recurrence without O' (Eq. 3 == Eq. 4)
 *   backward               Alg. 3 "Attn-QAT backward", with the two rules of
 *                          Sec. 2.3: P is re-quantized, D comes from O'
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - the block scale is stored as E4M3 (OCP "fn": bias 7, subnormals, max
 *     448, no infinity): s = RNE_E4M3(max|X| / 6), saturating at 448; a scale
 *     that rounds to 0 zeroes its block.  scale_mode 1 keeps Eq. 1 literally
 *     (s = max|X|/6 as an fp32 number) for diagnostics.
 *   - "round to the nearest FP4 value" is round-to-nearest-even on the real
 *     quotient |x|/s, saturating at 6.
 *   - P blocks are 16 consecutive keys aligned to absolute key indices that
 *     are multiples of 16 (32 and 32 in the MX format, scale_mode 2); masked and
 *     out-of-range keys count as 0.
 *   - key tiles of Bk keys are visited in increasing order; the running max
 *     used for quantizing P-tilde is the max over all tiles seen so far.
 *
 * MX variant (the OCP microscaling format named in Sec. 2.1 next to NVFP4: E2M1
 * elements, 32 per block, power-of-two E8M0 scale), same algorithms with
 *   - the block scale is the smallest power of two s with 6 s >= max|X| (the
 *     E8M0 counterpart of Eq. 1's s = max|X|/6: no element saturates), not below
 *     2^-126; a block of zeros gets 2^-126,
 *   - Q and K in blocks of 32 along d, P-tilde and V in blocks of 32 along the
 *     keys (aligned to absolute key indices that are multiples of 32), so that
 *     both products contract over the blocked axis.
 *
 * Parity status: every exported function below is pinned by the CPU tests
 * (format tables, closed forms, library attention with phi off, an independent
 * row-wise transcription with phi on, autograd of the unrolled STE graph).
 * Model-level claims of the paper (quality recovery) are parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ formats */

/* E2M1 magnitudes, index = low three bits of a code (Sec. 1: 15 distinct values, max 6). */
static const double E2M1[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double oracle_e2m1_value(int code)
{
    double v = E2M1[code & 7];
    return (code & 8) ? -v : v;
}

/* E4M3 value of a byte 0x00..0x7E (sign bit clear; 0x7F is NaN and never produced). */
double oracle_e4m3_value(int byte)
{
    int e = (byte >> 3) & 15, m = byte & 7;
    if (e == 0) return ldexp((double)m / 8.0, -6);
    return ldexp(1.0 + (double)m / 8.0, e - 7);
}

/* Byte of RNE_E4M3(amax / 6), saturating at 448 (byte 0x7E).
 * Decided on amax against 6 * midpoint, both exact in fp64, so the rounding
 * is that of the real quotient. */
int oracle_e4m3_from_amax(double amax)
{
    int i = 0;
    while (i < 0x7E) {
        double mid6 = 6.0 * 0.5 * (oracle_e4m3_value(i) + oracle_e4m3_value(i + 1));
        if (amax > mid6 || (amax == mid6 && (i & 1))) ++i; else break;
    }
    return i;
}

/* Magnitude index of RNE_E2M1(ax / s), ax >= 0, s > 0, saturating at 6.
 * Decided on ax against midpoint * s, exact in fp64. */
int oracle_e2m1_round(double ax, double s)
{
    int i = 0;
    while (i < 7) {
        double mid = 0.5 * (E2M1[i] + E2M1[i + 1]) * s;
        if (ax > mid || (ax == mid && (i & 1))) ++i; else break;
    }
    return i;
}

/* phi then phi^-1 on one block of n <= 16 values (Eq. 1, Eq. 2).
 * code[i] = sign<<3 | magnitude index; *scale is the block scale as a number,
 * *scale_byte its E4M3 byte (0 in scale_mode 1). */
static void phi_block(const double* x, int n, int scale_mode,
                      uint8_t* code, double* scale, uint8_t* scale_byte, double* xf)
{
    double amax = 0.0;
    for (int i = 0; i < n; ++i) { double a = fabs(x[i]); if (a > amax) amax = a; }
    double s; int sb = 0;
    if (scale_mode == 0) { sb = oracle_e4m3_from_amax(amax); s = oracle_e4m3_value(sb); }
    else                 { s = (double)(float)(amax / 6.0); }
    for (int i = 0; i < n; ++i) {
        int sign = signbit(x[i]) ? 8 : 0;
        int mag = (s > 0.0) ? oracle_e2m1_round(fabs(x[i]), s) : 0;
        if (code) code[i] = (uint8_t)(sign | mag);
        if (xf) xf[i] = (sign ? -1.0 : 1.0) * s * E2M1[mag];
    }
    if (scale) *scale = s;
    if (scale_byte) *scale_byte = (uint8_t)sb;
}

/* phi over the last axis of x[nrows, d] (blocks of 16 along d; d % 16 == 0).
 * packed[nrows, d/2]: element 2k in bits 3:0, element 2k+1 in bits 7:4.
 * scales[nrows, d/16] E4M3 bytes.  xf[nrows, d] = phi^-1(phi(x)).  Any output may be NULL. */
int oracle_phi(const float* x, long nrows, int d, int scale_mode,
               uint8_t* packed, uint8_t* scales, float* xf)
{
    if (!x || d < 16 || d % 16) return -1;
    #pragma omp parallel for schedule(static)
    for (long r = 0; r < nrows; ++r) {
        for (int c0 = 0; c0 < d; c0 += 16) {
            double xb[16], xfb[16], s; uint8_t code[16], sb;
            for (int i = 0; i < 16; ++i) xb[i] = (double)x[r * d + c0 + i];
            phi_block(xb, 16, scale_mode, code, &s, &sb, xfb);
            if (packed) for (int i = 0; i < 16; i += 2)
                packed[(r * d + c0 + i) / 2] = (uint8_t)(code[i] | (code[i + 1] << 4));
            if (scales) scales[r * (d / 16) + c0 / 16] = sb;
            if (xf) for (int i = 0; i < 16; ++i) xf[r * d + c0 + i] = (float)xfb[i];
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- MX format */

/* E8M0 byte (value 2^(byte-127)) of the smallest power of two s >= 2^-126 with 6 s >= amax.
 * 6 * 2^e is exact in fp64, so the comparison is that of the real numbers. */
int oracle_e8m0_from_amax(double amax)
{
    int e = -126;
    while (e < 127 && ldexp(6.0, e) < amax) ++e;
    return e + 127;
}

/* phi then phi^-1 on one MX block of n <= 32 values. */
static void phi_mx_block(const double* x, int n, uint8_t* code, uint8_t* scale_byte, double* xf)
{
    double amax = 0.0;
    for (int i = 0; i < n; ++i) { double a = fabs(x[i]); if (a > amax) amax = a; }
    int sb = oracle_e8m0_from_amax(amax);
    double s = ldexp(1.0, sb - 127);
    for (int i = 0; i < n; ++i) {
        int sign = signbit(x[i]) ? 8 : 0;
        int mag = oracle_e2m1_round(fabs(x[i]), s);
        if (code) code[i] = (uint8_t)(sign | mag);
        if (xf) xf[i] = (sign ? -1.0 : 1.0) * s * E2M1[mag];
    }
    if (scale_byte) *scale_byte = (uint8_t)sb;
}

/* MX phi over the last axis of x[nrows, n] in blocks of 32 (the last block may be short and is
 * padded with zeros).  With nb = ceil(n/32): packed[nrows, nb*16] (element 2k in bits 3:0),
 * scales[nrows, nb] E8M0 bytes, xf[nrows, n].  Any output may be NULL. */
int oracle_phi_mx(const float* x, long nrows, long n, uint8_t* packed, uint8_t* scales, float* xf)
{
    if (!x || n < 1) return -1;
    const long nb = (n + 31) / 32;
    #pragma omp parallel for schedule(static)
    for (long r = 0; r < nrows; ++r) {
        for (long b = 0; b < nb; ++b) {
            double xb[32], xfb[32]; uint8_t code[32], sb;
            const int m = (int)((n - b * 32 < 32) ? n - b * 32 : 32);
            for (int i = 0; i < 32; ++i) { xb[i] = i < m ? (double)x[r * n + b * 32 + i] : 0.0; }
            phi_mx_block(xb, 32, code, &sb, xfb);
            if (packed) for (int i = 0; i < 32; i += 2)
                packed[(r * nb + b) * 16 + i / 2] = (uint8_t)(code[i] | (code[i + 1] << 4));
            if (scales) scales[r * nb + b] = sb;
            if (xf) for (int i = 0; i < m; ++i) xf[r * n + b * 32 + i] = (float)xfb[i];
        }
    }
    return 0;
}

/* MXFP8 (E4M3 elements, 32 per block, E8M0 scale): the element format of the mixed recipe that keeps
 * FP4 for Q K^T and uses FP8 for P V (Sec. 2.5; scale_mode 3).  Same scale rule with E4M3's largest
 * value in place of 6: the smallest power of two s >= 2^-126 with 448 s >= max|X|. */
int oracle_e8m0_from_amax_fp8(double amax)
{
    int e = -126;
    while (e < 127 && ldexp(448.0, e) < amax) ++e;
    return e + 127;
}

/* Byte (sign clear) of RNE_E4M3(ax / s), ax >= 0, s a power of two, saturating at 448 (0x7E).
 * Decided on ax against midpoint * s, exact in fp64. */
int oracle_e4m3_round(double ax, double s)
{
    int lo = 0, hi = 0x7E;                      /* largest i with value(i) * s <= ax */
    while (lo < hi) {
        int mid = (lo + hi + 1) / 2;
        if (oracle_e4m3_value(mid) * s <= ax) lo = mid; else hi = mid - 1;
    }
    if (lo == 0x7E) return lo;
    double m = 0.5 * (oracle_e4m3_value(lo) + oracle_e4m3_value(lo + 1)) * s;
    if (ax > m || (ax == m && (lo & 1))) return lo + 1;
    return lo;
}

static void phi_mx8_block(const double* x, int n, uint8_t* code, uint8_t* scale_byte, double* xf)
{
    double amax = 0.0;
    for (int i = 0; i < n; ++i) { double a = fabs(x[i]); if (a > amax) amax = a; }
    int sb = oracle_e8m0_from_amax_fp8(amax);
    double s = ldexp(1.0, sb - 127);
    for (int i = 0; i < n; ++i) {
        int sign = signbit(x[i]) ? 0x80 : 0;
        int mag = oracle_e4m3_round(fabs(x[i]), s);
        if (code) code[i] = (uint8_t)(sign | mag);
        if (xf) xf[i] = (sign ? -1.0 : 1.0) * s * oracle_e4m3_value(mag);
    }
    if (scale_byte) *scale_byte = (uint8_t)sb;
}

/* MXFP8 phi over the last axis of x[nrows, n] in blocks of 32 (a short last block is zero padded).
 * With nb = ceil(n/32): codes[nrows, nb*32] E4M3 bytes, scales[nrows, nb] E8M0 bytes, xf[nrows, n]. */
int oracle_phi_mx8(const float* x, long nrows, long n, uint8_t* codes, uint8_t* scales, float* xf)
{
    if (!x || n < 1) return -1;
    const long nb = (n + 31) / 32;
    #pragma omp parallel for schedule(static)
    for (long r = 0; r < nrows; ++r) {
        for (long b = 0; b < nb; ++b) {
            double xb[32], xfb[32]; uint8_t code[32], sb;
            const int m = (int)((n - b * 32 < 32) ? n - b * 32 : 32);
            for (int i = 0; i < 32; ++i) { xb[i] = i < m ? (double)x[r * n + b * 32 + i] : 0.0; }
            phi_mx8_block(xb, 32, code, &sb, xfb);
            if (codes) for (int i = 0; i < 32; ++i) codes[(r * nb + b) * 32 + i] = code[i];
            if (scales) scales[r * nb + b] = sb;
            if (xf) for (int i = 0; i < m; ++i) xf[r * n + b * 32 + i] = (float)xfb[i];
        }
    }
    return 0;
}

/* ------------------------------------------------- two-level quantization of P */

/* SageAttention3's two-level scheme as Sec. 2.1 describes it and Sec. 3.2 switches on inside QAT
 * (scale_mode 4): every row of a P tile is first rescaled so that its maximum lands just below
 * 448 * 6 (the largest block scale times the largest element), then quantized as usual in NVFP4
 * blocks of 16.  Readings: a "row" is the 64 keys of one key tile (TWO_LEVEL_SPAN = B_k, the key
 * tile of the forward); the backward applies the same operator to the same aligned groups of 64
 * keys of the recomputed P (Sec. 2.3, "Matching the precision of P in the forward and backward
 * passes": the recomputation goes through the quantizer the forward used); the row factor is
 * rounded up to a power of two, s1 = the smallest 2^k with 2688 * 2^k >= max(rowmax, 2^-24), so that the rescale
 * is exact in every number format involved (the row maximum lands in (1344, 2688]) and rows
 * without any mass do not produce unbounded factors. */
#define TWO_LEVEL_SPAN 64
static double two_level_s1(double rowmax)
{
    double base = rowmax > ldexp(1.0, -24) ? rowmax : ldexp(1.0, -24);
    int k = -60;
    while (ldexp(2688.0, k) < base) ++k;
    return ldexp(1.0, k);
}
double oracle_two_level_s1(double rowmax) { return two_level_s1(rowmax); }

/* phi^-1(phi(.)) of n (a multiple of 16, <= 64) values of one row of a P tile with the two levels. */
static void phi_two_level(const double* P, int n, double* Pf)
{
    double rmax = 0.0;
    for (int k = 0; k < n; ++k) if (P[k] > rmax) rmax = P[k];
    const double s1 = two_level_s1(rmax);
    double P2[TWO_LEVEL_SPAN], Pf2[TWO_LEVEL_SPAN];
    for (int k = 0; k < n; ++k) P2[k] = P[k] / s1;                 /* exact: a power of two */
    for (int k = 0; k < n; k += 16) phi_block(P2 + k, 16, 0, NULL, NULL, NULL, Pf2 + k);
    for (int k = 0; k < n; ++k) Pf[k] = s1 * Pf2[k];
}

/* ---------------------------------------------------- formats of P-tilde in the P V product */

/* x (an fp32 value) rounded to bf16, nearest, ties to even: the "BF16" of the mixed recipes of Sec. 2.5
 * ("Bypassing the softmax bottleneck": NVFP4 Q K^T with BF16 or FP8 P V). */
static double bf16_rne(double x)
{
    float f = (float)x; uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* The format P-tilde takes before P V, chosen by scale_mode:
 *   0, 1  NVFP4 blocks of 16 keys (1: with the un-rounded fp32 scale of Eq. 1, diagnostics)
 *   2     MX FP4 blocks of 32 keys          3  MXFP8 blocks of 32 keys (mixed recipe FP4 Q K^T / FP8 P V)
 *   4     NVFP4 after the two-level row factor (the row is the whole tile: Bk = 64)
 *   5     bf16 (mixed recipe NVFP4 Q K^T / BF16 P V: P-tilde is not block-quantized at all) */
enum { PF_NVFP4 = 0, PF_MX = 1, PF_MXFP8 = 2, PF_TWO_LEVEL = 3, PF_BF16 = 4 };
static int p_format_of(int scale_mode)
{
    return scale_mode == 2 ? PF_MX : scale_mode == 3 ? PF_MXFP8 : scale_mode == 4 ? PF_TWO_LEVEL : scale_mode == 5 ? PF_BF16 : PF_NVFP4;
}

/* phi^-1(phi(.)) of one tile row of P-tilde: Pt[0..nk) are the visible keys, Pt[nk..Bk) are masked (0). */
static void quantize_p_row(int pf, int scale_mode, const double* Pt, int nk, int Bk, double* Pf)
{
    const int pb = (pf == PF_MX || pf == PF_MXFP8) ? 32 : 16;
    if (pf == PF_TWO_LEVEL) { phi_two_level(Pt, Bk, Pf); return; }
    if (pf == PF_BF16) { for (int k = 0; k < nk; ++k) Pf[k] = bf16_rne(Pt[k]); return; }
    for (int k = 0; k < nk; k += pb) {
        if (pf == PF_MXFP8)   phi_mx8_block(Pt + k, pb, NULL, NULL, Pf + k);
        else if (pf == PF_MX) phi_mx_block(Pt + k, pb, NULL, NULL, Pf + k);
        else                  phi_block(Pt + k, pb, scale_mode, NULL, NULL, NULL, Pf + k);
    }
}

/* ------------------------------------------------------------------ forward */

static double dot(const float* a, const float* b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += (double)a[c] * (double)b[c];
    return s;
}

/*
 * Alg. 2 for a list of query rows (rows are independent of each other and of Bq).
 * qf,kf,vf: Q^F, K^F, V^F (or the raw tensors when input quantization is off),
 *           [B,Hq,L,d] / [B,Hkv,L,d]; query head h reads kv head h / (Hq/Hkv).
 * rows:     nrows flat ids (b*Hq + h)*L + i, or NULL for all B*Hq*L rows in order.
 * Outputs per listed row: O[nrows,d], Op[nrows,d] (= O'), Lse[nrows];
 * Pdump[nrows, L] (optional) receives the dequantized P-tilde^F of each key as it
 * entered the O update (0 for masked keys).
 */
static int fwd_rows_impl(const float* qf, const float* kf, const float* vf,
                    int B, int Hq, int Hkv, long L, int d, int causal, int Bk,
                    int quant_p, int scale_mode,
                    long nrows, const long* rows,
                    double* O, double* Op, double* Lse, float* Pdump,
                    const uint8_t* bmask, int mbq, int mbk)
{
    /* Block-sparse attention (the datacenter inference kernel of Sec. 2.5 supports it, Sec. 5): bmask[B,Hq,ceil(L/mbq),ceil(L/mbk)],
     * a zero byte removes the whole block of mbq queries x mbk keys (mbk a multiple of Bk): its key tiles are not
     * visited.  A row with no key left gets O = 0 and L = -inf. */
    if (bmask && (mbq < 1 || mbk < Bk || mbk % Bk)) return -1;
    const long nqb = bmask ? (L + mbq - 1) / mbq : 0, nkb = bmask ? (L + mbk - 1) / mbk : 0;
    const int pf = p_format_of(scale_mode);
    const int pb = (pf == PF_MX || pf == PF_MXFP8) ? 32 : 16;    /* keys per P block */
    if (!qf || !kf || !vf || Hq % Hkv || Bk < pb || Bk % pb || d < 1) return -1;
    if (pf == PF_TWO_LEVEL && Bk != TWO_LEVEL_SPAN) return -1;
    const int G = Hq / Hkv;
    const double rs = 1.0 / sqrt((double)d);
    if (!rows) nrows = (long)B * Hq * L;
    int err = 0;
    #pragma omp parallel
    {
        double* S  = (double*)malloc(sizeof(double) * Bk);
        double* Pt = (double*)malloc(sizeof(double) * Bk);
        double* Pf = (double*)malloc(sizeof(double) * Bk);
        double* o  = (double*)malloc(sizeof(double) * d);
        double* op = (double*)malloc(sizeof(double) * d);
        if (!S || !Pt || !Pf || !o || !op) {
            #pragma omp atomic write
            err = 1;
        } else {
        #pragma omp for schedule(dynamic, 4)
        for (long n = 0; n < nrows; ++n) {
            long rid = rows ? rows[n] : n;
            long i = rid % L; long bh = rid / L; int h = (int)(bh % Hq); int b = (int)(bh / Hq);
            const float* qrow = qf + rid * d;
            const float* kh = kf + ((long)b * Hkv + h / G) * L * d;
            const float* vh = vf + ((long)b * Hkv + h / G) * L * d;
            double m = -INFINITY, l = 0.0;
            for (int c = 0; c < d; ++c) { o[c] = 0.0; op[c] = 0.0; }
            if (Pdump) for (long k = 0; k < L; ++k) Pdump[n * L + k] = 0.0f;
            long kend = causal ? i + 1 : L;           /* visible keys are [0, kend) */
            for (long k0 = 0; k0 < kend; k0 += Bk) {  /* tiles with no visible key change nothing */
                if (bmask && !bmask[(((long)b * Hq + h) * nqb + i / mbq) * nkb + k0 / mbk]) continue;
                int nk = (int)((kend - k0 < Bk) ? kend - k0 : Bk);
                double mt = -INFINITY;
                for (int k = 0; k < nk; ++k) {
                    S[k] = dot(qrow, kh + (k0 + k) * d, d) * rs;
                    if (S[k] > mt) mt = S[k];
                }
                double mnew = (m > mt) ? m : mt;
                double alpha = (m == -INFINITY) ? 0.0 : exp(m - mnew);
                double rowsum = 0.0;
                for (int k = 0; k < nk; ++k) {
                    Pt[k] = (double)(float)exp(S[k] - mnew);   /* fp32 softmax numerator */
                    rowsum += Pt[k];
                }
                for (int k = nk; k < Bk; ++k) Pt[k] = 0.0;      /* masked keys */
                if (quant_p) quantize_p_row(pf, scale_mode, Pt, nk, Bk, Pf);
                else for (int k = 0; k < nk; ++k) Pf[k] = Pt[k];
                l = alpha * l + rowsum;                          /* un-quantized P-tilde */
                m = mnew;
                for (int c = 0; c < d; ++c) { o[c] *= alpha; op[c] *= alpha; }
                for (int k = 0; k < nk; ++k) {
                    const float* vrow = vh + (k0 + k) * d;
                    for (int c = 0; c < d; ++c) {
                        o[c]  += Pf[k] * (double)vrow[c];
                        op[c] += Pt[k] * (double)vrow[c];
                    }
                    if (Pdump) Pdump[n * L + k0 + k] = (float)Pf[k];
                }
            }
            for (int c = 0; c < d; ++c) {
                if (O)  O[n * d + c]  = l > 0.0 ? o[c] / l : 0.0;
                if (Op) Op[n * d + c] = l > 0.0 ? op[c] / l : 0.0;
            }
            if (Lse) Lse[n] = l > 0.0 ? m + log(l) : -INFINITY;
        }
        }
        free(S); free(Pt); free(Pf); free(o); free(op);
    }
    return err ? -2 : 0;
}

/* scale_mode 2: the MX format (qf, kf, vf are then the MX fake-quantized tensors, V blocked along
 * the keys, and P-tilde is quantized in MX blocks of 32 keys).  scale_mode 3: the same with MXFP8
 * (E4M3 elements) for P-tilde (and, in the caller's vf, for V).  scale_mode 4: NVFP4 with the
 * two-level quantization of P-tilde (Bk must be 64).  scale_mode 5: P-tilde in bf16 (and, in the
 * caller's vf, V left as it is): NVFP4 Q K^T with BF16 P V.  Modes 3 and 5 are inference recipes: the
 * backward entry points refuse them. */
int oracle_fwd_rows(const float* qf, const float* kf, const float* vf,
                    int B, int Hq, int Hkv, long L, int d, int causal, int Bk,
                    int quant_p, int scale_mode,
                    long nrows, const long* rows,
                    double* O, double* Op, double* Lse, float* Pdump)
{
    return fwd_rows_impl(qf, kf, vf, B, Hq, Hkv, L, d, causal, Bk, quant_p, scale_mode,
                         nrows, rows, O, Op, Lse, Pdump, NULL, 0, 0);
}

/* The same with a block mask (see fwd_rows_impl). */
int oracle_fwd_rows_masked(const float* qf, const float* kf, const float* vf,
                           int B, int Hq, int Hkv, long L, int d, int causal, int Bk,
                           int quant_p, int scale_mode,
                           long nrows, const long* rows,
                           double* O, double* Op, double* Lse, float* Pdump,
                           const uint8_t* bmask, int mbq, int mbk)
{
    return fwd_rows_impl(qf, kf, vf, B, Hq, Hkv, L, d, causal, Bk, quant_p, scale_mode,
                         nrows, rows, O, Op, Lse, Pdump, bmask, mbq, mbk);
}

/* ----------------------------------------------------------------- backward */

/* Keys per P block: 16 (NVFP4), 32 in the MX format (scale_mode 2).  The mixed FP4/FP8 recipe (scale_mode 3) is an
 * inference recipe and has no backward: the entry points below refuse it. */
#define PB_MAX 32
static int pb_of(int scale_mode) { return scale_mode == 2 ? 32 : 16; }

/*
 * One query row against one aligned block of pb keys [k0, k0+pb): the inner
 * statements of Alg. 3.  nvis = number of keys of the block the row may see
 * (the rest are masked: P = 0), kend = end of the row's visible keys.  Returns P (fp32-rounded),
 * P^F and dS.
 */
/* Two-level P in the backward: the row factor of the aligned group of TWO_LEVEL_SPAN keys (the forward's
 * tile row) that holds block k0 (keys >= kend are masked: P = 0). */
static double span_s1(const float* qrow, double lse, const float* kh, long k0, long kend, int d, double rs)
{
    long s0 = k0 - k0 % TWO_LEVEL_SPAN;
    double rmax = 0.0;
    for (long k = s0; k < s0 + TWO_LEVEL_SPAN && k < kend; ++k) {
        double p = (double)(float)exp(dot(qrow, kh + k * d, d) * rs - lse);
        if (p > rmax) rmax = p;
    }
    return two_level_s1(rmax);
}

static void bwd_block(const float* qrow, const float* dorow, double lse, double D,
                      const float* kh, const float* vh, long k0, int nvis, long kend, int d, double rs,
                      int quant_p, int scale_mode, double* P, double* Pf, double* dS)
{
    const int pb = pb_of(scale_mode);
    for (int k = 0; k < pb; ++k) {
        if (k < nvis) {
            double s = dot(qrow, kh + (k0 + k) * d, d) * rs;
            P[k] = (double)(float)exp(s - lse);
        } else P[k] = 0.0;
    }
    if (quant_p && scale_mode == 4) {
        const double s1 = span_s1(qrow, lse, kh, k0, kend, d, rs);
        double P2[16], Pf2[16];
        for (int k = 0; k < 16; ++k) P2[k] = P[k] / s1;
        phi_block(P2, 16, 0, NULL, NULL, NULL, Pf2);
        for (int k = 0; k < 16; ++k) Pf[k] = s1 * Pf2[k];
    }
    else if (quant_p && scale_mode == 2) phi_mx_block(P, pb, NULL, NULL, Pf);
    else if (quant_p) phi_block(P, pb, scale_mode, NULL, NULL, NULL, Pf);
    else for (int k = 0; k < pb; ++k) Pf[k] = P[k];
    for (int k = 0; k < pb; ++k) {
        if (k < nvis) {
            double dP = dot(dorow, vh + (k0 + k) * d, d);
            dS[k] = P[k] * (dP - D) * rs;        /* fp32 P, not P^F (Sec. 2.3) */
        } else dS[k] = 0.0;
    }
}

static int nvis_of(long k0, long kend, int pb)
{
    long n = kend - k0;
    return (int)(n < 0 ? 0 : (n > pb ? pb : n));
}

/*
 * Alg. 3 on the whole problem.  Lse[B,Hq,L], Op[B,Hq,L,d] are the forward's L
 * and O'.  dQ[B,Hq,L,d], dK/dV[B,Hkv,L,d] (summed over the query heads of a group).
 */
int oracle_bwd(const float* qf, const float* kf, const float* vf, const float* dO,
               const double* Lse, const double* Op,
               int B, int Hq, int Hkv, long L, int d, int causal,
               int quant_p, int scale_mode,
               double* dQ, double* dK, double* dV)
{
    if (!qf || !kf || !vf || !dO || !Lse || !Op || Hq % Hkv) return -1;
    if (scale_mode == 3 || scale_mode == 5) return -3;
    const int G = Hq / Hkv;
    const double rs = 1.0 / sqrt((double)d);
    const int pb = pb_of(scale_mode);
    memset(dQ, 0, sizeof(double) * (size_t)B * Hq * L * d);
    memset(dK, 0, sizeof(double) * (size_t)B * Hkv * L * d);
    memset(dV, 0, sizeof(double) * (size_t)B * Hkv * L * d);
    #pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < (long)B * Hkv; ++u) {      /* one kv head: no two threads share dK/dV */
        const float* kh = kf + u * L * d;
        const float* vh = vf + u * L * d;
        int b = (int)(u / Hkv), hk = (int)(u % Hkv);
        for (int g = 0; g < G; ++g) {
            long bh = (long)b * Hq + hk * G + g;
            for (long i = 0; i < L; ++i) {
                long rid = bh * L + i;
                const float* qrow = qf + rid * d; const float* dorow = dO + rid * d;
                double D = 0.0;                                   /* D = rowsum(dO o O') */
                for (int c = 0; c < d; ++c) D += (double)dorow[c] * Op[rid * d + c];
                long kend = causal ? i + 1 : L;
                for (long k0 = 0; k0 < kend; k0 += pb) {
                    double P[PB_MAX], Pf[PB_MAX], dS[PB_MAX];
                    int nv = nvis_of(k0, kend, pb);
                    bwd_block(qrow, dorow, Lse[rid], D, kh, vh, k0, nv, kend, d, rs,
                              quant_p, scale_mode, P, Pf, dS);
                    for (int k = 0; k < nv; ++k) {
                        long kr = (u * L + k0 + k) * d;
                        for (int c = 0; c < d; ++c) {
                            dV[kr + c] += Pf[k] * (double)dorow[c];
                            dQ[rid * d + c] += dS[k] * (double)kh[(k0 + k) * d + c];
                            dK[kr + c] += dS[k] * (double)qrow[c];
                        }
                    }
                }
            }
        }
    }
    return 0;
}

/* dQ for a list of query rows (flat ids as in oracle_fwd_rows); Lse_rows[nrows]
 * and Op_rows[nrows,d] belong to the same list. */
int oracle_bwd_dq_rows(const float* qf, const float* kf, const float* vf, const float* dO,
                       int B, int Hq, int Hkv, long L, int d, int causal,
                       int quant_p, int scale_mode,
                       long nrows, const long* rows,
                       const double* Lse_rows, const double* Op_rows, double* dQ_rows)
{
    if (!rows || Hq % Hkv) return -1;
    if (scale_mode == 3 || scale_mode == 5) return -3;
    (void)B;
    const int G = Hq / Hkv;
    const double rs = 1.0 / sqrt((double)d);
    const int pb = pb_of(scale_mode);
    #pragma omp parallel for schedule(dynamic, 1)
    for (long n = 0; n < nrows; ++n) {
        long rid = rows[n]; long i = rid % L; long bh = rid / L;
        int h = (int)(bh % Hq), b = (int)(bh / Hq);
        const float* kh = kf + ((long)b * Hkv + h / G) * L * d;
        const float* vh = vf + ((long)b * Hkv + h / G) * L * d;
        const float* qrow = qf + rid * d; const float* dorow = dO + rid * d;
        double D = 0.0;
        for (int c = 0; c < d; ++c) D += (double)dorow[c] * Op_rows[n * d + c];
        for (int c = 0; c < d; ++c) dQ_rows[n * d + c] = 0.0;
        long kend = causal ? i + 1 : L;
        for (long k0 = 0; k0 < kend; k0 += pb) {
            double P[PB_MAX], Pf[PB_MAX], dS[PB_MAX];
            int nv = nvis_of(k0, kend, pb);
            bwd_block(qrow, dorow, Lse_rows[n], D, kh, vh, k0, nv, kend, d, rs,
                      quant_p, scale_mode, P, Pf, dS);
            for (int k = 0; k < nv; ++k)
                for (int c = 0; c < d; ++c)
                    dQ_rows[n * d + c] += dS[k] * (double)kh[(k0 + k) * d + c];
        }
    }
    return 0;
}

/* dK and dV for a list of key rows of ONE kv head (b, hk).  Lse_grp[G,L] and
 * Op_grp[G,L,d] hold L and O' of every query row of the G = Hq/Hkv query heads
 * that read this kv head.  Pf_dump (optional) [nkeys, G, L] receives P^F[i, key]. */
int oracle_bwd_dkdv_keys(const float* qf, const float* kf, const float* vf, const float* dO,
                         int B, int Hq, int Hkv, long L, int d, int causal,
                         int quant_p, int scale_mode,
                         int b, int hk, long nkeys, const long* keys,
                         const double* Lse_grp, const double* Op_grp,
                         double* dK_keys, double* dV_keys, float* Pf_dump)
{
    if (!keys || Hq % Hkv || b < 0 || b >= B || hk < 0 || hk >= Hkv) return -1;
    if (scale_mode == 3 || scale_mode == 5) return -3;
    const int G = Hq / Hkv;
    const double rs = 1.0 / sqrt((double)d);
    const int pb = pb_of(scale_mode);
    const float* kh = kf + ((long)b * Hkv + hk) * L * d;
    const float* vh = vf + ((long)b * Hkv + hk) * L * d;
    /* D for every query row of the group */
    double* Dg = (double*)malloc(sizeof(double) * (size_t)G * L);
    if (!Dg) return -2;
    #pragma omp parallel for schedule(static)
    for (long r = 0; r < (long)G * L; ++r) {
        long rid = ((long)b * Hq + hk * G) * L + r;
        double D = 0.0;
        for (int c = 0; c < d; ++c) D += (double)dO[rid * d + c] * Op_grp[r * d + c];
        Dg[r] = D;
    }
    #pragma omp parallel for schedule(dynamic, 1)
    for (long n = 0; n < nkeys; ++n) {
        long key = keys[n]; long k0 = key - key % pb; int kk = (int)(key - k0);
        for (int c = 0; c < d; ++c) { dK_keys[n * d + c] = 0.0; dV_keys[n * d + c] = 0.0; }
        for (int g = 0; g < G; ++g) {
            for (long i = 0; i < L; ++i) {
                long kend = causal ? i + 1 : L;
                if (Pf_dump) Pf_dump[(n * G + g) * L + i] = 0.0f;
                if (key >= kend) continue;
                long rid = ((long)b * Hq + hk * G + g) * L + i;
                double P[PB_MAX], Pf[PB_MAX], dS[PB_MAX];
                bwd_block(qf + rid * d, dO + rid * d, Lse_grp[g * L + i], Dg[g * L + i],
                          kh, vh, k0, nvis_of(k0, kend, pb), kend, d, rs, quant_p, scale_mode, P, Pf, dS);
                for (int c = 0; c < d; ++c) {
                    dV_keys[n * d + c] += Pf[kk] * (double)dO[rid * d + c];
                    dK_keys[n * d + c] += dS[kk] * (double)qf[rid * d + c];
                }
                if (Pf_dump) Pf_dump[(n * G + g) * L + i] = (float)Pf[kk];
            }
        }
    }
    free(Dg);
    return 0;
}

/* dK and dV contributions of a LIST of query rows, for all keys (Alg. 3 with the outer
 * sums restricted to the listed rows).  Because dP, D and therefore dS, and dV = P^F^T dO,
 * are linear in dO, this equals the full backward whenever dO is zero outside the list.
 * rows: flat ids; Lse_rows[nrows], Op_rows[nrows,d] belong to the list.
 * dK, dV [B,Hkv,L,d] are overwritten. */
int oracle_bwd_rows_dkdv(const float* qf, const float* kf, const float* vf, const float* dO,
                         int B, int Hq, int Hkv, long L, int d, int causal,
                         int quant_p, int scale_mode,
                         long nrows, const long* rows,
                         const double* Lse_rows, const double* Op_rows,
                         double* dK, double* dV)
{
    if (!rows || Hq % Hkv) return -1;
    if (scale_mode == 3 || scale_mode == 5) return -3;
    const int G = Hq / Hkv;
    const double rs = 1.0 / sqrt((double)d);
    const int pb = pb_of(scale_mode);
    memset(dK, 0, sizeof(double) * (size_t)B * Hkv * L * d);
    memset(dV, 0, sizeof(double) * (size_t)B * Hkv * L * d);
    for (long n = 0; n < nrows; ++n) {              /* rows one after another ... */
        long rid = rows[n]; long i = rid % L; long bh = rid / L;
        int h = (int)(bh % Hq), b = (int)(bh / Hq);
        long u = (long)b * Hkv + h / G;
        const float* kh = kf + u * L * d; const float* vh = vf + u * L * d;
        const float* qrow = qf + rid * d; const float* dorow = dO + rid * d;
        double D = 0.0;
        for (int c = 0; c < d; ++c) D += (double)dorow[c] * Op_rows[n * d + c];
        long kend = causal ? i + 1 : L;
        long nblk = (kend + pb - 1) / pb;
        #pragma omp parallel for schedule(static)   /* ... key blocks in parallel: disjoint dK/dV rows */
        for (long kb = 0; kb < nblk; ++kb) {
            long k0 = kb * pb;
            double P[PB_MAX], Pf[PB_MAX], dS[PB_MAX];
            int nv = nvis_of(k0, kend, pb);
            bwd_block(qrow, dorow, Lse_rows[n], D, kh, vh, k0, nv, kend, d, rs, quant_p, scale_mode, P, Pf, dS);
            for (int k = 0; k < nv; ++k) {
                long kr = (u * L + k0 + k) * d;
                for (int c = 0; c < d; ++c) {
                    dV[kr + c] += Pf[k] * (double)dorow[c];
                    dK[kr + c] += dS[k] * (double)qrow[c];
                }
            }
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
