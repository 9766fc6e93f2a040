// phi of Eq. 1 / Eq. 2 (Sec. 2.1) as a streaming kernel, plus the layout copies the
// attention kernels read: the first line of Alg. 1 (phi(Q), phi(K), phi(V)) and of
// Alg. 2 (Q^F, K^F, V^F).  HBM-bandwidth bound.
//
// One thread owns one block of 16 consecutive d-elements (32 bytes in).  A workgroup
// covers 64 sequence positions; the optional transposed copy goes through LDS so that
// both the row-major and the transposed stores are 16-byte vectors.
#include "common.hpp"
#include "kernels.hpp"

namespace aq {

// Position p (0..15) inside a group of 16 sequence positions of a transposed copy holds
// sequence index perm16(p): quads 1 and 2 are exchanged.  A lane of a 32x32x16 MFMA
// accumulator owns sequence indices {0-3, 8-11} (lanes 0-31) or {4-7, 12-15} (lanes
// 32-63) of such a group, so with this order its 8 values pair with one contiguous
// 16-byte run of the transposed operand.
__host__ __device__ inline int perm16(int p) { return (p & ~12) | ((p & 4) << 1) | ((p & 8) >> 1); }

// phi of one block of 16 values that are bf16 numbers (Eq. 1): the E4M3 scale s and the 16 E2M1 codes, element 2k in the low
// nibble of byte k of {clo, chi}.
// RNE of the real quotient x / s without a division per element (ten vector instructions each, which bound the streaming
// kernels).  |x| has 8 significant bits and s has 4, so a quotient that is not on a rounding boundary of the E2M1 grid is at
// least 2^-9 (relative) away from it, and one that is on a boundary (a tie) has at most 3 significant bits.  x * (1/s) with the
// approximate reciprocal is within 2^-21 of the quotient; rounding that product to 12 significant bits puts a tie back on its
// boundary exactly and moves nothing else across one (it moves a value by at most 2^-12).  The rounding to E2M1 itself
// (nearest, ties to even, saturating at 6, sign kept) then is the hardware conversion, two elements per instruction, which
// leaves the codes packed as the public layout wants them.
__device__ inline void phi_block16_bf16(const float (&v)[16], float& s, uint32_t& clo, uint32_t& chi)
{
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
    s = block_scale_exact(amax);
    const float inv_s = s > 0.0f ? __builtin_amdgcn_rcpf(s) : 0.0f;      // s = 0: every quotient 0, every code 0
    auto snap = [](float r) __attribute__((always_inline)) {
        return __uint_as_float((__float_as_uint(r) + 0x800u) & 0xFFFFF000u);
    };
    clo = 0; chi = 0;
#define AQ_PAIR(W, PR, SEL) W = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(W, snap(v[2 * (PR)] * inv_s), snap(v[2 * (PR) + 1] * inv_s), 1.0f, SEL)
    AQ_PAIR(clo, 0, 0); AQ_PAIR(clo, 1, 1); AQ_PAIR(clo, 2, 2); AQ_PAIR(clo, 3, 3);
    AQ_PAIR(chi, 4, 0); AQ_PAIR(chi, 5, 1); AQ_PAIR(chi, 6, 2); AQ_PAIR(chi, 7, 3);
#undef AQ_PAIR
}

// The 16 values of a block from its codes and its scale (exact: <= 6 significant bits).
__device__ inline void dequant_block16(uint32_t clo, uint32_t chi, float s, float (&xf)[16])
{
    typedef float float2v __attribute__((ext_vector_type(2)));
#define AQ_BACK(W, PR, SEL) { const float2v cv = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(W, 1.0f, SEL); xf[2 * (PR)] = cv[0] * s; xf[2 * (PR) + 1] = cv[1] * s; }
    AQ_BACK(clo, 0, 0) AQ_BACK(clo, 1, 1) AQ_BACK(clo, 2, 2) AQ_BACK(clo, 3, 3)
    AQ_BACK(chi, 4, 0) AQ_BACK(chi, 5, 1) AQ_BACK(chi, 6, 2) AQ_BACK(chi, 7, 3)
#undef AQ_BACK
}

// The NVFP4 KV cache: a page holds 128 consecutive positions of one sequence for all kv heads; per kv head, in this order,
// K codes [128][D/2], K scale bytes [128][D/16], V codes [128][D/2], V scale bytes [128][D/16]: the public layout of
// attnqat_quantize cut into pages.  Blocks run along d, so positions are independent of each other: a sequence grows by
// writing its new positions only.
__host__ __device__ inline size_t nvfp4_page_head_bytes(int D) { return (size_t)2 * 128 * (D / 2 + D / 16); }
struct PagedSrc {
    const unsigned char* cache; const int* table; const int* kv_lens;
    int max_pages, num_pages, Hkv, which;          // which: 0 the K part, 1 the V part
};
// Codes and scale byte of block cb of position l (nullptr for a page id outside the cache).
__device__ inline const unsigned char* nvfp4_page_part(const unsigned char* cache, int page, int num_pages, int Hkv, int h, int D, int which) {
    if (page < 0 || page >= num_pages) return nullptr;
    return cache + ((size_t)page * Hkv + h) * nvfp4_page_head_bytes(D) + (size_t)which * 128 * (D / 2 + D / 16);
}

// PACKED (with QUANT = false): the input is not x but an already quantized tensor, codes [BH, L, D/2] and E4M3 scale bytes
// [BH, L, D/16] in the public layout of attnqat_quantize (read through `codes` and `scales`); the kernel writes the
// dequantized layout copies, the same values the quantizing variant writes for the tensor those codes came from.
// PAGED (with PACKED): the quantized tensor is the K or the V part of the pages of an NVFP4 KV cache; bh = sequence * Hkv + kv
// head, position l of sequence b is slot l % 128 of page table[b][l / 128], positions from kv_lens[b] on read as zeros, and
// L is the capacity max_pages * 128 that the copies are laid out for.
template <bool QUANT, bool OUT_F16, bool PACKED = false, bool PAGED = false>
__global__ __launch_bounds__(256) void prep_kernel(
    const uint16_t* __restrict__ x, int L, int Lp, int D,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint16_t* __restrict__ xf_pub,
    uint16_t* __restrict__ xr, uint16_t* __restrict__ xt, const float* __restrict__ sub, PagedSrc ps)
{
    static_assert(!(QUANT && PACKED), "a packed input is already quantized");
    static_assert(!PAGED || PACKED, "pages hold quantized tensors");
    __shared__ uint16_t tile[64][128 + 2];
    const int bh = blockIdx.y;
    const int l0 = blockIdx.x * 64;
    const int nb = D / 16;                       // 16-element blocks per row
    const size_t in_base = (size_t)bh * L * D;
    int Lseq = L;
    const unsigned char* page_part[PAGED ? 1 : 1] = {nullptr};
    if constexpr (PAGED) {
        const int b = bh / ps.Hkv;
        Lseq = max(0, min(ps.kv_lens[b], L));
        if (l0 >= Lseq) return;                  // key tiles that start beyond the sequence are never read
        // a workgroup's 64 positions lie in one page
        page_part[0] = nvfp4_page_part(ps.cache, ps.table[(size_t)b * ps.max_pages + (l0 >> 7)], ps.num_pages, ps.Hkv, bh % ps.Hkv, D, ps.which);
    }

    for (int blk = threadIdx.x; blk < 64 * nb; blk += 256) {
        const int row = blk / nb, cb = blk % nb;
        const int l = l0 + row;
        float v[16];
        if (PACKED) {
            const unsigned char* cp = nullptr; const unsigned char* sp = nullptr;
            if constexpr (PAGED) {
                if (l < Lseq && page_part[0]) {
                    cp = page_part[0] + (size_t)(l & 127) * (D / 2) + cb * 8;
                    sp = page_part[0] + (size_t)128 * (D / 2) + (size_t)(l & 127) * nb + cb;
                }
            } else if (l < L) {
                cp = codes + ((size_t)bh * L + l) * (D / 2) + cb * 8;
                sp = scales + ((size_t)bh * L + l) * nb + cb;
            }
            if (cp) {
                const uint2v cw = *reinterpret_cast<const uint2v*>(cp);
                // E4M3 byte -> value: the hardware conversion (OCP E4M3, subnormals kept), byte 0 of the operand
                dequant_block16(cw[0], cw[1], __builtin_amdgcn_cvt_scalef32_f32_fp8((uint32_t)*sp, 1.0f, 0), v);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = 0.0f;
            }
        } else if (l < L) {
            const uint4v* src = reinterpret_cast<const uint4v*>(x + in_base + (size_t)l * D + cb * 16);
            uint4v a = src[0], b = src[1];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i]         = __uint_as_float(a[i] << 16);
                v[2 * i + 1]     = __uint_as_float(a[i] & 0xFFFF0000u);
                v[8 + 2 * i]     = __uint_as_float(b[i] << 16);
                v[8 + 2 * i + 1] = __uint_as_float(b[i] & 0xFFFF0000u);
            }
            if (sub) {                      // K smoothing: minus the token mean of the channel, an fp32 subtraction.
                // The inputs of phi then have 24 significant bits: the two "IEEE division == real quotient" arguments
                // below hold up to a double rounding that can move a value sitting within 2^-24 of a rounding boundary.
                const float* sp = sub + (size_t)bh * D + cb * 16;
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] -= sp[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = 0.0f;
        }

        float xf[16];
        if (QUANT) {
            float s;
            uint32_t clo = 0, chi = 0;
            if (sub) {
                float amax = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
                s = block_scale_exact(amax);
                // (inputs with 24 significant bits, after the K smoothing subtraction: IEEE division and the grid rounding
                //  of common.hpp; the short cut below relies on bf16 inputs)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t sign = __float_as_uint(v[i]) >> 31;
                    float q = 0.0f;
                    if (s > 0.0f) {
                        float r = fabsf(v[i]) / s;
                        r = r < 6.0f ? r : 6.0f;
                        q = rne_e2m1_grid(r);
                    }
                    const uint32_t code = (sign << 3) | e2m1_index_of(q);
                    if (i < 8) clo |= code << (4 * i); else chi |= code << (4 * (i - 8));
                    const float d = q * s;                   // exact: <= 6 significant bits
                    xf[i] = sign ? -d : d;
                }
            } else {
                phi_block16_bf16(v, s, clo, chi);
                dequant_block16(clo, chi, s, xf);
            }
            if (l < L) {
                if (codes) {
                    uint2v c2; c2[0] = clo; c2[1] = chi;
                    *reinterpret_cast<uint2v*>(codes + ((size_t)bh * L + l) * (D / 2) + cb * 8) = c2;
                }
            }
            if (scales) {
                // four neighbouring blocks of a row (four neighbouring lanes: nb is 4 or 8 and a wave starts at a multiple
                // of 64 blocks) write their scale bytes as one dword; rows beyond L take part in the exchange and write nothing
                uint32_t sb = e4m3_byte_of(s);
                sb |= (uint32_t)__shfl_down((int)sb, 1) << 8;
                sb |= (uint32_t)__shfl_down((int)sb, 2) << 16;
                if (l < L && (cb & 3) == 0) *reinterpret_cast<uint32_t*>(scales + ((size_t)bh * L + l) * nb + cb) = sb;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) xf[i] = v[i];
        }

        if (xf_pub && l < L) {                           // public bf16 copy, un-padded
            uint4v o0, o1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o0[i] = pack_bf16x2_rne(xf[2 * i], xf[2 * i + 1]);
                o1[i] = pack_bf16x2_rne(xf[8 + 2 * i], xf[8 + 2 * i + 1]);
            }
            uint4v* dst = reinterpret_cast<uint4v*>(xf_pub + in_base + (size_t)l * D + cb * 16);
            dst[0] = o0; dst[1] = o1;
        }
        // workspace copies: fp16 or bf16; both hold s*c exactly
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            w[i] = OUT_F16 ? pack_f16x2(xf[2 * i], xf[2 * i + 1]) : pack_bf16x2_rne(xf[2 * i], xf[2 * i + 1]);
        if (xr) {                                        // row-major, rows padded to Lp with zeros
            uint4v o0, o1;
#pragma unroll
            for (int i = 0; i < 4; ++i) { o0[i] = w[i]; o1[i] = w[4 + i]; }
            uint4v* dst = reinterpret_cast<uint4v*>(xr + ((size_t)bh * Lp + l) * D + cb * 16);
            dst[0] = o0; dst[1] = o1;
        }
        if (xt) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                tile[row][cb * 16 + 2 * i]     = (uint16_t)(w[i] & 0xFFFFu);
                tile[row][cb * 16 + 2 * i + 1] = (uint16_t)(w[i] >> 16);
            }
        }
    }
    if (xt) {
        __syncthreads();
        // transposed copy [bh][c][Lp]: 8 positions (16 bytes) per store
        for (int ch = threadIdx.x; ch < D * 8; ch += 256) {
            const int c = ch >> 3, kc = ch & 7;
            uint4v o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p0 = kc * 8 + 2 * j, p1 = p0 + 1;
                const int r0 = (p0 & ~15) | perm16(p0 & 15), r1 = (p1 & ~15) | perm16(p1 & 15);
                o[j] = (uint32_t)tile[r0][c] | ((uint32_t)tile[r1][c] << 16);
            }
            *reinterpret_cast<uint4v*>(xt + ((size_t)bh * D + c) * Lp + l0 + kc * 8) = o;
        }
    }
}

// Writer of the NVFP4 KV cache: phi of n new positions pos0 .. pos0 + n - 1 of one sequence, k and v [Hkv, n, D] bf16, into
// the pages page_ids[pos / 128] (the sequence's page list).  The slots between the last new position and the end of its page
// are cleared (codes and scales 0: they read as zeros until the sequence grows into them).  A page id outside [0, num_pages)
// is left out.  One thread per block of 16 elements; grid (64-row groups, Hkv, 2: K then V).
template <int D>
__global__ __launch_bounds__(256) void kv_page_write_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, int n, int pos0, int Hkv,
    unsigned char* __restrict__ cache, int num_pages, const int* __restrict__ page_ids)
{
    constexpr int nb = D / 16;
    const int h = blockIdx.y, which = blockIdx.z;
    const uint16_t* x = (which ? v : k) + (size_t)h * n * D;
    const int rows_total = ((pos0 + n + 127) & ~127) - pos0;
    for (int blk = threadIdx.x; blk < 64 * nb; blk += 256) {
        const int row = blockIdx.x * 64 + blk / nb, cb = blk % nb;
        float s = 0.0f;
        uint32_t clo = 0, chi = 0;
        if (row < n) {
            const uint4v* src = reinterpret_cast<const uint4v*>(x + (size_t)row * D + cb * 16);
            const uint4v a = src[0], b = src[1];
            float val[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                val[2 * i]         = __uint_as_float(a[i] << 16);
                val[2 * i + 1]     = __uint_as_float(a[i] & 0xFFFF0000u);
                val[8 + 2 * i]     = __uint_as_float(b[i] << 16);
                val[8 + 2 * i + 1] = __uint_as_float(b[i] & 0xFFFF0000u);
            }
            phi_block16_bf16(val, s, clo, chi);
        }
        // the scale bytes of four neighbouring blocks of a row as one dword (rows beyond the page end take part and write nothing)
        uint32_t sb = e4m3_byte_of(s);
        sb |= (uint32_t)__shfl_down((int)sb, 1) << 8;
        sb |= (uint32_t)__shfl_down((int)sb, 2) << 16;
        if (row >= rows_total) continue;
        const int pos = pos0 + row;
        unsigned char* part = const_cast<unsigned char*>(nvfp4_page_part(cache, page_ids[pos >> 7], num_pages, Hkv, h, D, which));
        if (!part) continue;
        uint2v c2; c2[0] = clo; c2[1] = chi;
        *reinterpret_cast<uint2v*>(part + (size_t)(pos & 127) * (D / 2) + cb * 8) = c2;
        if ((cb & 3) == 0) *reinterpret_cast<uint32_t*>(part + (size_t)128 * (D / 2) + (size_t)(pos & 127) * nb + cb) = sb;
    }
}

size_t nvfp4_page_bytes(int Hkv, int D) { return (size_t)Hkv * nvfp4_page_head_bytes(D); }

int launch_kv_page_write(const void* k, const void* v, int Hkv, int n, int D, int pos0,
                         void* cache, int num_pages, const int* page_ids, hipStream_t st)
{
    if (Hkv > 65535 || (D != 64 && D != 128) || n < 1 || pos0 < 0) return -1;
    const int rows_total = ((pos0 + n + 127) & ~127) - pos0;
    dim3 grid((rows_total + 63) / 64, Hkv, 2);
    if (D == 128) hipLaunchKernelGGL((kv_page_write_kernel<128>), grid, dim3(256), 0, st, (const uint16_t*)k, (const uint16_t*)v, n, pos0, Hkv,
                                     (unsigned char*)cache, num_pages, page_ids);
    else          hipLaunchKernelGGL((kv_page_write_kernel<64>), grid, dim3(256), 0, st, (const uint16_t*)k, (const uint16_t*)v, n, pos0, Hkv,
                                     (unsigned char*)cache, num_pages, page_ids);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// The layout copies of the forward (K row-major fp16, or V transposed fp16) from the pages of B sequences; the copies are laid
// out for max_pages * 128 positions per sequence.
int launch_unpack_pages(const void* cache, const int* page_table, const int* kv_lens, int B, int Hkv, int max_pages, int num_pages,
                        int D, int which, void* xr, void* xt, hipStream_t st)
{
    const int L = max_pages * 128, Lp = round_up(L, kRowPad);
    if ((size_t)B * Hkv > 65535) return -1;
    PagedSrc ps{(const unsigned char*)cache, page_table, kv_lens, max_pages, num_pages, Hkv, which};
    hipLaunchKernelGGL((prep_kernel<false, true, true, true>), dim3(Lp / 64, B * Hkv), dim3(256), 0, st, (const uint16_t*)nullptr, L, Lp, D,
                       (uint8_t*)nullptr, (uint8_t*)nullptr, (uint16_t*)nullptr, (uint16_t*)xr, (uint16_t*)xt, (const float*)nullptr, ps);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Token mean of every channel, for K smoothing: fp64 partial sums of NCHUNK row ranges, then their sum in a fixed
// order, divided by L and rounded to fp32.  Deterministic; x [BH, L, D] bf16.
constexpr int kMeanChunks = 32;
template <int D>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const uint16_t* __restrict__ x, int L, double* __restrict__ part)
{
    constexpr int NS = 256 / D;                       // row slices per block
    __shared__ double red[256];
    const int bh = blockIdx.y, ch = blockIdx.x, c = threadIdx.x % D, sl = threadIdx.x / D;
    const int per = (L + kMeanChunks - 1) / kMeanChunks;
    const int r0 = ch * per, r1 = min(L, r0 + per);
    const uint16_t* src = x + (size_t)bh * L * D + c;
    double acc = 0.0;
    for (int r = r0 + sl; r < r1; r += NS) acc += (double)bf16_to_f32(src[(size_t)r * D]);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (sl == 0) {
        double t = red[c];
#pragma unroll
        for (int i = 1; i < NS; ++i) t += red[i * D + c];
        part[((size_t)bh * kMeanChunks + ch) * D + c] = t;
    }
}
__global__ void colmean_kernel(const double* __restrict__ part, int L, int D, float* __restrict__ mean)
{
    const int bh = blockIdx.x, c = threadIdx.x;
    double t = 0.0;
    for (int ch = 0; ch < kMeanChunks; ++ch) t += part[((size_t)bh * kMeanChunks + ch) * D + c];
    mean[(size_t)bh * D + c] = (float)(t / (double)L);
}

size_t colmean_scratch_bytes(int BH, int D) { return (size_t)BH * kMeanChunks * D * sizeof(double); }

int launch_colmean(const void* x, int BH, int L, int D, double* scratch, float* mean, hipStream_t st)
{
    if (BH > 65535 || (D != 64 && D != 128)) return -1;
    if (D == 128) hipLaunchKernelGGL((colsum_partial_kernel<128>), dim3(kMeanChunks, BH), dim3(256), 0, st, (const uint16_t*)x, L, scratch);
    else          hipLaunchKernelGGL((colsum_partial_kernel<64>), dim3(kMeanChunks, BH), dim3(256), 0, st, (const uint16_t*)x, L, scratch);
    if (hipGetLastError() != hipSuccess) return -1;
    hipLaunchKernelGGL(colmean_kernel, dim3(BH), dim3(D), 0, st, (const double*)scratch, L, D, mean);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <bool QUANT, bool OUT_F16>
static int launch_prep_t(const void* x, int BH, int L, int D, uint8_t* codes, uint8_t* scales,
                         void* xf_pub, void* xr, void* xt, const float* sub, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    dim3 grid(Lp / 64, BH);
    hipLaunchKernelGGL((prep_kernel<QUANT, OUT_F16>), grid, dim3(256), 0, st,
                       (const uint16_t*)x, L, Lp, D, codes, scales, (uint16_t*)xf_pub,
                       (uint16_t*)xr, (uint16_t*)xt, sub, PagedSrc{});
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_unpack(const uint8_t* codes, const uint8_t* scales, int BH, int L, int D, bool out_f16, void* xr, void* xt, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    dim3 grid(Lp / 64, BH);
    if (out_f16) hipLaunchKernelGGL((prep_kernel<false, true, true>), grid, dim3(256), 0, st, (const uint16_t*)nullptr, L, Lp, D,
                                    const_cast<uint8_t*>(codes), const_cast<uint8_t*>(scales), (uint16_t*)nullptr, (uint16_t*)xr, (uint16_t*)xt, (const float*)nullptr, PagedSrc{});
    else         hipLaunchKernelGGL((prep_kernel<false, false, true>), grid, dim3(256), 0, st, (const uint16_t*)nullptr, L, Lp, D,
                                    const_cast<uint8_t*>(codes), const_cast<uint8_t*>(scales), (uint16_t*)nullptr, (uint16_t*)xr, (uint16_t*)xt, (const float*)nullptr, PagedSrc{});
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_prep(const void* x, int BH, int L, int D, bool quant, bool out_f16,
                uint8_t* codes, uint8_t* scales, void* xf_pub, void* xr, void* xt, hipStream_t st, const float* sub)
{
    if (quant) return out_f16 ? launch_prep_t<true, true>(x, BH, L, D, codes, scales, xf_pub, xr, xt, sub, st)
                              : launch_prep_t<true, false>(x, BH, L, D, codes, scales, xf_pub, xr, xt, sub, st);
    return out_f16 ? launch_prep_t<false, true>(x, BH, L, D, codes, scales, xf_pub, xr, xt, sub, st)
                   : launch_prep_t<false, false>(x, BH, L, D, codes, scales, xf_pub, xr, xt, sub, st);
}

}  // namespace aq
