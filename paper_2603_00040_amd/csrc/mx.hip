// MX variant of the quantizer and of the inference forward (Alg. 1) on the scaled FP4 MFMA of gfx950.
// (The MX training forward and backward are variants of the 16-bit kernels in fwd.hip and bwd.hip.)
//
// Format (the OCP microscaling FP4 that Sec. 2.1 names beside NVFP4): E2M1 elements in blocks of 32
// with one power-of-two E8M0 scale, the smallest 2^e (e >= -126) with 6 * 2^e >= max|X|: the
// power-of-two counterpart of Eq. 1, no element saturates.  Q and K are blocked along d, P-tilde and
// V along the keys, so both products of Alg. 1 contract over the blocked axis and run on
// v_mfma_scale_f32_32x32x64_f8f6f4 with the FP4 codes and the scale bytes as they are: there is no
// dequantization anywhere, and phi(P-tilde) is one exponent extraction plus the hardware converts.
//
// Operand layout of that instruction with FP4 on both sides (checked on the device against a
// scalar evaluation): lane l holds row (A) or column (B) l % 32 and the 32 contraction indices
// 32 * (l / 32) .. + 31 as 32 nibbles in 4 registers, low nibble first, plus one scale byte for
// exactly those 32 indices: one MX block per lane.
//
//   S^T[key, query]  = K codes (A, from LDS) x Q codes (B, registers), contraction over d
//   O^T[d, query]   += V^T codes (A, from LDS) x P-tilde codes (B, registers), contraction over keys
//
// Mixed recipe (Sec. 2.5: FP4 for Q K^T, FP8 for P V): the FP8PV variants keep Q and K in MXFP4 and hold V and
// P-tilde in MXFP8 (E4M3 elements, the same blocks of 32 keys and E8M0 scales; scale = smallest 2^e with
// 448 * 2^e >= max|X|).  The P.V product then runs the same instruction with FP8 operands, whose layout differs
// (measured): the 32 bytes of lane l are contraction indices 16 (l/32) .. + 15 and 32 + 16 (l/32) .. + 15, and the
// scale of indices 32 b .. + 31 comes from lane l % 32 + 32 b.
//
// The rows of the two S^T products of a 64-key tile are assigned to keys so that the 32 accumulator
// registers of a lane are the 32 consecutive keys 32 * (lane / 32) .. + 31 of the tile: one P block,
// whose maximum, scale and codes never leave the lane, and whose 4 code registers already are the
// B operand of the P.V product.
#include "common.hpp"
#include "kernels.hpp"

namespace aq {

#ifndef AQ_DECODE_NP
#define AQ_DECODE_NP 1     // pages per iteration of the decode kernel (4 waves per page)
#endif

typedef int int8v __attribute__((ext_vector_type(8)));

// 32 values -> 4 registers of E2M1 codes (value i in nibble i), RNE on v / scale, saturating.
__device__ inline uint4v mx_codes32(const float (&v)[32], float scale) {
    uint4v c;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t r = 0u;
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * w + 0], v[8 * w + 1], scale, 0);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * w + 2], v[8 * w + 3], scale, 1);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * w + 4], v[8 * w + 5], scale, 2);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * w + 6], v[8 * w + 7], scale, 3);
        c[w] = r;
    }
    return c;
}

__device__ inline float e2m1_value_of(uint32_t code) {
    const uint32_t m = code & 7u;
    const float v = m < 2u ? 0.5f * (float)m : __uint_as_float(((m >> 1) + 126u) << 23 | (m & 1u) << 22);
    return (code & 8u) ? -v : v;
}

// Bytes of one 64-key record of a kv head: K operands, V^T operands, K scales, V scales.
__host__ __device__ constexpr int mx_rec_bytes(int D, bool fp8v = false) { return 2 * (D / 64) * 1024 + (D / 32) * (fp8v ? 2048 : 1024) + 512; }

// 32 values -> 8 registers of E4M3 bytes (value i in byte i), RNE on v / scale; |v| / scale <= 448 by the scale rule.
typedef short short2v __attribute__((ext_vector_type(2)));
__device__ inline void mx_codes32_fp8(const float (&v)[32], float scale, uint32_t (&c)[8]) {
#pragma unroll
    for (int w = 0; w < 8; ++w) {
        short2v r = {0, 0};
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, v[4 * w + 0], v[4 * w + 1], scale, false);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, v[4 * w + 2], v[4 * w + 3], scale, true);
        c[w] = __builtin_bit_cast(uint32_t, r);
    }
}
__device__ inline float e4m3_value_of(uint32_t byte) {
    const uint32_t e = (byte >> 3) & 15u, m = byte & 7u;
    const float v = e == 0u ? (float)m * 0.001953125f : __uint_as_float((e + 120u) << 23 | m << 20);
    return (byte & 0x80u) ? -v : v;
}

// Where the 64-key record `tile` of kv head `head` lives.  Contiguous: records of a head one after another.  Paged (a
// KV cache): a page holds two records (128 keys) of every kv head, page_ids[tile / 2] names the page of this sequence.
// A page id outside [0, num_pages) gives null: the writer leaves that record out instead of touching memory outside the cache.
__device__ inline unsigned char* mx_record_of(unsigned char* base, const int* page_ids, int num_pages, int head, int nheads, int Lp, int tile, int rec_bytes) {
    if (page_ids) {
        const int page = page_ids[tile >> 1];
        if (page < 0 || page >= num_pages) return nullptr;
        return base + (((size_t)page * nheads + head) * 2 + (tile & 1)) * rec_bytes;
    }
    return base + ((size_t)head * (Lp / 64) + tile) * rec_bytes;
}

// Row of S^T product t (0/1) that holds key kk (0..63) of a tile, and the lane half that ends up owning it:
// the accumulator register r of a lane in half h is row 8 (r/4) + 4 h + r % 4; key 32 h + 16 t + r goes there.
__device__ inline int mx_srow_of_key(int kk) { const int w = kk & 15; return 8 * (w >> 2) + 4 * (kk >> 5) + (w & 3); }

// ---------------------------------------------------------------------------------------------
// phi along d (blocks of 32).  One thread per block.
//   MODE 0: public layout   codes [rows, D/2], scales [rows, D/32], optional bf16 xf
//   MODE 1: Q operands      ops [rows/32, D/64, 64 lanes, 16 B], sc [rows/32, 64 lanes] (byte ks)
//   MODE 2: K part of the kv records
//   MODE 3: K records of the training forward (16-bit P V, scores on the FP4 instruction): per 64-key tile
//           mx_ktrain_rec_bytes(D) bytes = ops [2 blocks of 32 keys][D/64][64 lanes][16 B] with the keys of a block in their
//           natural order as operand rows (so that the score tile has the accumulator layout of the 16-bit kernels), then
//           per lane one dword of scale bytes (byte = block * D/64 + ks), padded to a whole KiB
template <int D, int MODE, bool FP8V = false /* MODE 2: records whose V part is FP8 */>
__global__ __launch_bounds__(256) void mx_quant_d_kernel(
    const uint16_t* __restrict__ x, int L, int Lp, unsigned char* __restrict__ codes, unsigned char* __restrict__ scales,
    uint16_t* __restrict__ xf, const int* __restrict__ page_ids, int num_pages)
{
    constexpr int NB = D / 32, KS = D / 64;
    const int bh = blockIdx.y;
    const int gid = blockIdx.x * 256 + threadIdx.x;
    const int row = gid / NB, blk = gid % NB;
    const int rows_out = MODE == 0 ? L : Lp;
    if (row >= rows_out) return;
    float v[32];
    if (row < L) {
        const uint4v* src = reinterpret_cast<const uint4v*>(x + ((size_t)bh * L + row) * D + blk * 32);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4v a = src[j];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[8 * j + 2 * i]     = __uint_as_float(a[i] << 16);
                v[8 * j + 2 * i + 1] = __uint_as_float(a[i] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = 0.0f;
    }
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
    const uint32_t byte = e8m0_of_amax(amax);
    const float s = e8m0_as_f32(byte);
    const uint4v c = mx_codes32(v, s);
    if (MODE == 0) {
        if (codes) *reinterpret_cast<uint4v*>(codes + ((size_t)bh * L + row) * (D / 2) + blk * 16) = c;
        if (scales) scales[((size_t)bh * L + row) * NB + blk] = (unsigned char)byte;
        if (xf) {
            uint4v o[4];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t w = c[i >> 2] >> (8 * (i & 3));
                // code * 2^e: at most 2 significant bits, exact in bf16 whenever it is a normal number
                const uint32_t lo = f32_to_bf16_rne(e2m1_value_of(w & 15u) * s), hi = f32_to_bf16_rne(e2m1_value_of((w >> 4) & 15u) * s);
                o[i >> 2][i & 3] = lo | (hi << 16);
            }
            uint4v* dst = reinterpret_cast<uint4v*>(xf + ((size_t)bh * L + row) * D + blk * 32);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = o[j];
        }
    } else if (MODE == 1) {
        const int g = row >> 5, ks = blk >> 1, lane = (blk & 1) * 32 + (row & 31);
        const size_t grp = (size_t)bh * (Lp / 32) + g;
        *reinterpret_cast<uint4v*>(codes + ((grp * KS + ks) * 64 + lane) * 16) = c;
        scales[(grp * 64 + lane) * 4 + ks] = (unsigned char)byte;
        if (KS == 1) { scales[(grp * 64 + lane) * 4 + 1] = 1; }
        if (ks == 0) { scales[(grp * 64 + lane) * 4 + 2] = 1; scales[(grp * 64 + lane) * 4 + 3] = 1; }
    } else if (MODE == 3) {
        constexpr int REC = mx_ktrain_rec_bytes(D), KOPS = 2 * KS * 1024;
        const int tile = row >> 6, kk = row & 63, kb = kk >> 5;
        const int ks = blk >> 1, lane = (blk & 1) * 32 + (kk & 31);
        unsigned char* rec = codes + ((size_t)bh * (Lp / 64) + tile) * REC;
        *reinterpret_cast<uint4v*>(rec + ((kb * KS + ks) * 64 + lane) * 16) = c;
        rec[KOPS + lane * 4 + kb * KS + ks] = (unsigned char)byte;
        if (KS == 1 && kb == 0) { rec[KOPS + lane * 4 + 2] = 1; rec[KOPS + lane * 4 + 3] = 1; }
    } else {
        constexpr int REC = mx_rec_bytes(D, FP8V), KOPS = 2 * KS * 1024, VOPS = NB * (FP8V ? 2048 : 1024);
        const int tile = row >> 6, kk = row & 63, t = (kk >> 4) & 1;
        const int ks = blk >> 1, lane = (blk & 1) * 32 + mx_srow_of_key(kk);
        unsigned char* rec = mx_record_of(codes, page_ids, num_pages, bh, (int)gridDim.y, Lp, tile, REC);
        if (!rec) return;
        *reinterpret_cast<uint4v*>(rec + ((t * KS + ks) * 64 + lane) * 16) = c;
        rec[KOPS + VOPS + lane * 4 + t * KS + ks] = (unsigned char)byte;
        if (KS == 1 && t == 0) { rec[KOPS + VOPS + lane * 4 + 2] = 1; rec[KOPS + VOPS + lane * 4 + 3] = 1; }
    }
}

// phi along the sequence axis (blocks of 32 positions, zero padded): how V is blocked.
// One thread per (block of 32 positions, d index); x [BH, L, D].  FP8: E4M3 elements (one byte each) instead of E2M1.
//   MODE 0: public layout  codes [BH, D, Lc/2] (FP8: [BH, D, Lc]), scales [BH, D, Lc/32] with Lc = round_up(L, 32);
//           optional bf16 xf [BH, L, D]
//   MODE 2: V part of the kv records (FP8: two 1 KiB halves per d-block, bytes 0-15 and 16-31 of every lane)
template <int D, int MODE, bool FP8>
__global__ __launch_bounds__(D) void mx_quant_l_kernel(
    const uint16_t* __restrict__ x, int L, int Lp, unsigned char* __restrict__ codes, unsigned char* __restrict__ scales,
    uint16_t* __restrict__ xf, const int* __restrict__ page_ids, int num_pages)
{
    constexpr int KS = D / 64, MT = D / 32;
    const int bh = blockIdx.y, kb = blockIdx.x, dd = threadIdx.x;
    const uint16_t* src = x + (size_t)bh * L * D + dd;
    float v[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int l = kb * 32 + i;
        v[i] = l < L ? bf16_to_f32(src[(size_t)l * D]) : 0.0f;
    }
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
    const uint32_t byte = FP8 ? e8m0_of_amax_fp8(amax) : e8m0_of_amax(amax);
    const float s = e8m0_as_f32(byte);
    uint32_t c[8];
    if constexpr (FP8) {
        mx_codes32_fp8(v, s, c);
    } else {
        const uint4v c4 = mx_codes32(v, s);
#pragma unroll
        for (int i = 0; i < 4; ++i) { c[i] = c4[i]; c[4 + i] = 0u; }
    }
    constexpr int NW = FP8 ? 8 : 4;                 // code registers per block
    if (MODE == 0) {
        const int Lc = round_up(L, 32);
        if (codes) {
            uint4v* dst = reinterpret_cast<uint4v*>(codes + (((size_t)bh * D + dd) * (Lc / 32) + kb) * (4 * NW));
#pragma unroll
            for (int i = 0; i < NW / 4; ++i) { uint4v o; o[0] = c[4 * i]; o[1] = c[4 * i + 1]; o[2] = c[4 * i + 2]; o[3] = c[4 * i + 3]; dst[i] = o; }
        }
        if (scales) scales[((size_t)bh * D + dd) * (Lc / 32) + kb] = (unsigned char)byte;
        if (xf) {
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int l = kb * 32 + i;
                const float val = FP8 ? e4m3_value_of((c[i >> 2] >> (8 * (i & 3))) & 255u) : e2m1_value_of((c[i >> 3] >> (4 * (i & 7))) & 15u);
                if (l < L) xf[((size_t)bh * L + l) * D + dd] = f32_to_bf16_rne(val * s);
            }
        }
    } else {
        constexpr int REC = mx_rec_bytes(D, FP8), KOPS = 2 * KS * 1024, VOPS = MT * (FP8 ? 2048 : 1024);
        const int tile = kb >> 1, lane = (kb & 1) * 32 + (dd & 31), mt = dd >> 5;
        unsigned char* rec = mx_record_of(codes, page_ids, num_pages, bh, (int)gridDim.y, Lp, tile, REC);
        if (!rec) return;
        if constexpr (FP8) {
            // FP8 operands: registers 0-3 of lane (row, h) are contraction indices 16 h .. + 15, registers 4-7 are
            // 32 + 16 h .. + 15, and the scale of indices 32 b .. + 31 is taken from lane (row, b): the two halves of
            // this block of 32 keys go to the two lane halves, in the register group of the block
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                uint4v o; o[0] = c[4 * i]; o[1] = c[4 * i + 1]; o[2] = c[4 * i + 2]; o[3] = c[4 * i + 3];
                *reinterpret_cast<uint4v*>(rec + KOPS + ((mt * 2 + (kb & 1)) * 64 + i * 32 + (dd & 31)) * 16) = o;
            }
        } else {
            uint4v o; o[0] = c[0]; o[1] = c[1]; o[2] = c[2]; o[3] = c[3];
            *reinterpret_cast<uint4v*>(rec + KOPS + (mt * 64 + lane) * 16) = o;
        }
        rec[KOPS + VOPS + 256 + lane * 4 + mt] = (unsigned char)byte;
        if (MT == 2 && mt == 0) { rec[KOPS + VOPS + 256 + lane * 4 + 2] = 1; rec[KOPS + VOPS + 256 + lane * 4 + 3] = 1; }
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 1 on the MX operands.  A workgroup of 4 waves owns 128 query rows of one head, a wave 32 of
// them, a lane one row and one of the two 32-key blocks of every 64-key tile (B_k = 64).
// kv records arrive in stages of two tiles, copied global->LDS directly into a ring of three stage
// buffers; one barrier per stage.  The S^T products of tile j+1 are issued before the softmax of
// tile j, so the matrix unit works under the wave's own vector instructions.
// PAGED: the kv records come from a KV cache (pages of 128 keys = one stage per kv head, located through
// page_table [B, max_pages]), every sequence has its own number of keys kv_lens[b] >= L, and the L queries are the
// LAST positions of the sequence.  lq_inner: the rows of a head are the G query heads of a kv group one after another,
// lq_inner positions each (L = G * lq_inner; a kv head's queries are contiguous in [B,Hq,Lq,d], so grouped-query
// heads with few positions share one tile and one pass over the pages); lq_inner == L: plain rows.  Under the causal
// mask the query at position i of its head sees keys 0 .. kv_len - lq_inner + i.
//
// KVM == 2, block-sparse attention on contiguous kv records: the workgroup visits only the 128-key blocks listed for its
// 128 query rows (page_table then is the list [B*Hq*ceil(L/128), max_pages] of block indices in increasing order and
// kv_lens the number of entries per row of that list); a row that ends up without any key gets O = 0 and L = -inf.
template <int D, bool CAUSAL, bool FP8PV, int KVM /* 0 contiguous, 1 paged KV cache, 2 block-sparse */>
__global__ __launch_bounds__(256, 2) void fwd_mx_kernel(
    const unsigned char* __restrict__ qops, const uint32_t* __restrict__ qsc, const unsigned char* __restrict__ kv,
    uint16_t* __restrict__ O, float* __restrict__ lse, int L, int Lp, int Hq, int G, float c /* log2(e)/sqrt(d) */,
    const int* __restrict__ page_table, const int* __restrict__ kv_lens, int max_pages, int num_pages, int lq_inner)
{
    constexpr int KS = D / 64, MT = D / 32;
    constexpr bool PAGED = KVM == 1, SPARSE = KVM == 2;
    constexpr int KOPS = 2 * KS * 1024, VOPS = MT * (FP8PV ? 2048 : 1024), REC = mx_rec_bytes(D, FP8PV), STAGE = 2 * REC, NCH = STAGE / 1024;
    static_assert(STAGE % 1024 == 0, "a stage is a whole number of 1 KiB wave copies");
    extern __shared__ __align__(16) unsigned char smem[];          // 3 stage buffers

    const int nqt = Lp / 128;
    int bh, qt;
    head_tile_of_block(blockIdx.x, gridDim.x / nqt, nqt, bh, qt);
    if (CAUSAL) qt = nqt - 1 - qt;                                 // longest rows first
    const int b = bh / Hq, h = bh % Hq;
    const int bhkv = b * (Hq / G) + h / G;
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row0_w = qt * 128 + wave * 32;
    const int q_row = row0_w + ln;
    const int wave_qmax = row0_w + 31;

    // Q operands of this lane: codes of its row for d-slots 64 ks + 32 hf .. + 31, scale bytes by ks
    uint4v qop[KS];
    const size_t grp = (size_t)bh * (Lp / 32) + (row0_w >> 5);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = *reinterpret_cast<const uint4v*>(qops + ((grp * KS + ks) * 64 + lane) * 16);
    uint32_t qs = qsc[grp * 64 + lane];

    const int Lk = PAGED ? __builtin_amdgcn_readfirstlane(kv_lens[b]) : L;      // keys of this sequence
    const int koff = PAGED ? Lk - lq_inner : 0;                    // key index of position 0's diagonal
    const bool packed = PAGED && lq_inner != L;                    // several heads' positions in this tile
    const int nkt_all = PAGED ? min((Lk + 63) / 64, 2 * max_pages) : (Lk + 63) / 64;   // never past the page table
    // block-sparse: the blocks of this workgroup's row of the list, and the first key of the block visited s-th
    const int* blk_row = SPARSE ? page_table + ((size_t)bh * nqt + qt) * max_pages : nullptr;
    const int nblk = SPARSE ? min(max(__builtin_amdgcn_readfirstlane(kv_lens[(size_t)bh * nqt + qt]), 0), max_pages) : 0;
    auto blk_of = [&](int s) __attribute__((always_inline)) -> int {
        return min(max(__builtin_amdgcn_readfirstlane(blk_row[s]), 0), Lp / 128 - 1);      // a bad entry reads a wrong block, never outside
    };
    const int nkt = SPARSE ? 2 * nblk
                  : (CAUSAL && !packed) ? min((koff + qt * 128 + 128 + 63) / 64, nkt_all) : nkt_all;   // tiles this workgroup visits
    const int nst = (nkt + 1) / 2;
    auto k0_of = [&](int j) __attribute__((always_inline)) -> int { return SPARSE ? blk_of(j >> 1) * 128 + (j & 1) * 64 : j * 64; };
    const unsigned char* kv_head = kv + (size_t)bhkv * (Lp / 64) * REC;
    const int Hkv = Hq / G;
    auto issue_stage = [&](int s) __attribute__((always_inline)) {
        const unsigned char* src = kv_head + (size_t)(SPARSE ? blk_of(s) : s) * STAGE;
        if constexpr (PAGED) {
            int page = __builtin_amdgcn_readfirstlane(page_table[(size_t)b * max_pages + s]);
            page = min(max(page, 0), num_pages - 1);               // a bad table entry reads a wrong page, never outside the cache
            src = kv + ((size_t)page * Hkv + (h / G)) * STAGE;
        }
        unsigned char* dst = smem + (s % 3) * STAGE;
        for (int i = wave; i < NCH; i += 4) async_copy16(src, (uint32_t)(i * 1024 + lane * 16), dst + i * 1024);
    };
    auto rec_of = [&](int j) __attribute__((always_inline)) -> const unsigned char* {
        return smem + ((j >> 1) % 3) * STAGE + (j & 1) * REC;
    };

    floatx16 o[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mt][i] = 0.0f;
    float m = -INFINITY, lsum = 0.0f;

    auto as8 = [](const uint4v& x) __attribute__((always_inline)) -> int8v {
        int8v r = {(int)x[0], (int)x[1], (int)x[2], (int)x[3], 0, 0, 0, 0};
        return r;
    };
    // S^T of one tile: product t covers keys {16 t .. 16 t + 15} of both 32-key blocks
    auto scores = [&](const unsigned char* rec, floatx16 (&s)[2]) __attribute__((always_inline)) {
        const uint32_t ksc = lds_read4(rec + KOPS + VOPS + lane * 4);
        uint4v a[2][KS];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[t][ks] = lds_read16(rec + ((t * KS + ks) * 64 + lane) * 16);
        // (a constant zero accumulator is encoded in the instruction: no registers to clear)
        const floatx16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0][0]), as8(qop[0]), zero, 4, 4, 0, ksc, 0, qs);
        s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1][0]), as8(qop[0]), zero, 4, 4, KS, ksc, 0, qs);
        if constexpr (KS == 2) {
            s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0][1]), as8(qop[1]), s[0], 4, 4, 1, ksc, 1, qs);
            s[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1][1]), as8(qop[1]), s[1], 4, 4, 3, ksc, 1, qs);
        }
    };
    // online softmax of one tile (Alg. 1 inner loop), phi of this lane's P-tilde block, O += V^F^T P-tilde^F
    auto softmax_pv = [&](int j, const unsigned char* rec, floatx16 (&s)[2]) __attribute__((always_inline)) {
        const int k0 = k0_of(j);
        const bool need_mask = (k0 + 64 > Lk) || (CAUSAL && k0 + 63 > koff + (packed ? 0 : row0_w));
        if (__builtin_expect(need_mask, 0)) {
            const int klim = CAUSAL ? min(Lk - 1, koff + (packed ? q_row % lq_inner : q_row)) : Lk - 1;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (k0 + 32 * hf + 16 * t + i > klim) s[t][i] = -INFINITY;
        }
        float mp[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) mp[t] = max_raw(s[0][t], s[1][t]);
#pragma unroll
        for (int i = 4; i < 16; ++i) mp[i & 3] = max_nc(max_nc(mp[i & 3], s[0][i]), s[1][i]);
        const float mown = max_nc(max_nc(mp[0], mp[1]), max_nc(mp[2], mp[3]));      // maximum of this lane's block
        const float mnew = max_nc(m, xhalf_max(mown));
        // (block-sparse: the first blocks a row meets may lie entirely in its causal future; until it has seen a key
        //  its maximum is -inf, and a finite stand-in keeps the two expressions below free of inf - inf)
        const float mref = (SPARSE && mnew == -INFINITY) ? 0.0f : mnew;
        const float alpha = __builtin_amdgcn_exp2f((m - mref) * c);
        const float ms = mref * c;
        m = mnew;
        float p[32];
        float rp[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[16 * t + i] = __builtin_amdgcn_exp2f(fmaf(s[t][i], c, -ms));
                rp[i & 3] += p[16 * t + i];
            }
        lsum = lsum * alpha + ((rp[0] + rp[1]) + (rp[2] + rp[3]));                  // un-quantized P-tilde
        // block maximum of P-tilde: exp2 of the block's largest score, the same instructions on the same inputs
        const float amax = __builtin_amdgcn_exp2f(fmaf(mown, c, -ms));
        const uint32_t pbyte = FP8PV ? e8m0_of_amax_fp8(amax) : e8m0_of_amax(amax);
        uint32_t pc[8];
        if constexpr (FP8PV) {
            // E4M3 bytes of this lane's block, then the exchange that the FP8 operand layout asks for: registers 0-3 of
            // lane (row, h) hold keys 16 h .. + 15 of the tile and registers 4-7 keys 32 + 16 h .. + 15, so the lower
            // half-wave hands the second half of its block to the upper one and takes the first half of the upper's
            uint32_t own[8];
            mx_codes32_fp8(p, e8m0_as_f32(pbyte), own);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                auto r = __builtin_amdgcn_permlane32_swap(own[i], own[4 + i], false, false);
                pc[i] = r[0]; pc[4 + i] = r[1];
            }
        } else {
            const uint4v c4 = mx_codes32(p, e8m0_as_f32(pbyte));
#pragma unroll
            for (int i = 0; i < 4; ++i) { pc[i] = c4[i]; pc[4 + i] = 0u; }
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0, 0)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[mt][i] *= alpha;
        }
        const uint32_t vsc = lds_read4(rec + KOPS + VOPS + 256 + lane * 4);
        const int8v pb = {(int)pc[0], (int)pc[1], (int)pc[2], (int)pc[3], (int)pc[4], (int)pc[5], (int)pc[6], (int)pc[7]};
        if constexpr (FP8PV) {
            int8v va[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const uint4v lo = lds_read16(rec + KOPS + ((2 * mt) * 64 + lane) * 16), hi = lds_read16(rec + KOPS + ((2 * mt + 1) * 64 + lane) * 16);
                va[mt] = int8v{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
            o[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[0], pb, o[0], 0, 0, 0, vsc, 0, pbyte);
            o[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[1], pb, o[1], 0, 0, 1, vsc, 0, pbyte);
            if constexpr (MT == 4) {
                o[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[2], pb, o[2], 0, 0, 2, vsc, 0, pbyte);
                o[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[3], pb, o[3], 0, 0, 3, vsc, 0, pbyte);
            }
        } else {
            uint4v va[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) va[mt] = lds_read16(rec + KOPS + (mt * 64 + lane) * 16);
            o[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[0]), pb, o[0], 4, 4, 0, vsc, 0, pbyte);
            o[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[1]), pb, o[1], 4, 4, 1, vsc, 0, pbyte);
            if constexpr (MT == 4) {
                o[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[2]), pb, o[2], 4, 4, 2, vsc, 0, pbyte);
                o[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[3]), pb, o[3], 4, 4, 3, vsc, 0, pbyte);
            }
        }
    };
    auto wave_sees = [&](int j) __attribute__((always_inline)) -> bool { return !CAUSAL || packed || k0_of(j) <= koff + wave_qmax; };
    // One tile: at odd j the next stage becomes visible (and the buffer two stages back becomes free).
    auto tile_step = [&](int j, floatx16 (&scur)[2], floatx16 (&snext)[2]) __attribute__((always_inline)) {
        if (j & 1) {
            __builtin_amdgcn_s_waitcnt(0);                 // this wave's part of stage (j+1)/2 is in LDS
            __builtin_amdgcn_s_barrier();                  // ... everyone's is, and everyone is past tile j-1
            if ((j >> 1) + 2 < nst) issue_stage((j >> 1) + 2);
        }
        if (j + 1 < nkt && wave_sees(j + 1)) scores(rec_of(j + 1), snext);
        if (wave_sees(j)) softmax_pv(j, rec_of(j), scur);
    };

    issue_stage(0);
    if (nst > 1) issue_stage(1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qop[ks]));
    asm volatile("" : "+v"(qs));
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    floatx16 sa[2], sb[2];
    scores(rec_of(0), sa);
    for (int j = 0; j < nkt; j += 2) {
        tile_step(j, sa, sb);
        if (j + 1 < nkt) tile_step(j + 1, sb, sa);
    }

    // ---- epilogue: O /= l, L = m + log l
    const float l = xhalf_sum(lsum);
    const float inv_l = ((PAGED || SPARSE) && !(l > 0.0f)) ? 0.0f : 1.0f / l;         // a row without keys: O = 0, L = -inf
    if (q_row < L) {
        const size_t row = (size_t)bh * L + q_row;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int d0 = 32 * mt + 8 * t + 4 * hf;
                uint2v w;
                w[0] = pack_bf16x2_rne(o[mt][4 * t] * inv_l, o[mt][4 * t + 1] * inv_l);
                w[1] = pack_bf16x2_rne(o[mt][4 * t + 2] * inv_l, o[mt][4 * t + 3] * inv_l);
                *reinterpret_cast<uint2v*>(O + row * D + d0) = w;
            }
        if (hf == 0) lse[row] = m * (c * 0.6931471805599453f) + logf(l);   // m is in raw q.k units
    }
}

// ---------------------------------------------------------------------------------------------
// Decode form of the paged forward: at most 32 query rows per (sequence, kv head) — one position, or a few, of the G
// query heads of a group — against a long sequence.  fwd_mx_kernel would leave three of its four waves without rows
// and walk the pages with one; here the waves of a workgroup share the KEYS: an iteration takes NP pages (a page: two
// 64-key tiles), and wave w takes the product t = w % 2 of tile T = (w / 2) % 2 of page w / 4 of the iteration, i.e.
// keys {32 hf + 16 t .. + 15} of that tile (16 of each of its two 32-key blocks), for all 32 rows.  What Alg. 1 makes
// sequential is only the running maximum, and that needs no more than the waves' partial row maxima of S: they go
// through LDS once per iteration, after which every wave knows the maximum after each of the 2 NP tiles and the largest
// score of its two blocks (exp2 of it, by the same instructions as that element's P-tilde, is the block's amax, so both
// waves of a block derive the same scale).  Each wave then quantizes its 16 keys per row against the maximum after ITS
// tile, exactly as the tile order of Alg. 1 prescribes, and accumulates its own O and l against its own reference
// maximum; the partial results are brought to the final maximum and added at the end.
template <int D, bool CAUSAL, int NP /* pages per iteration: 4 NP waves */>
__global__ __launch_bounds__(256 * NP, NP == 1 ? 2 : 1) void fwd_mx_decode_kernel(
    const unsigned char* __restrict__ qops, const uint32_t* __restrict__ qsc, const unsigned char* __restrict__ kv,
    uint16_t* __restrict__ O, float* __restrict__ lse, int L /* rows, <= 32 */, int Hq, int G, float c /* log2(e)/sqrt(d) */,
    const int* __restrict__ page_table, const int* __restrict__ kv_lens, int max_pages, int num_pages, int lq_inner)
{
    constexpr int KS = D / 64, MT = D / 32, NW = 4 * NP;
    constexpr int NIT = NP == 1 ? 4 : NP == 2 ? 3 : 2;   // iterations whose pages the LDS ring holds (NIT - 1 of them in flight)
    constexpr int NR = NIT * NP;                     // ... in pages
    constexpr int KOPS = 2 * KS * 1024, VOPS = MT * 1024, REC = mx_rec_bytes(D, false), STAGE = 2 * REC, NCH = STAGE / 1024;
    constexpr int NV = MT * 16 + 1;                  // floats per lane in the final reduction
    static_assert(STAGE % 1024 == 0 && NR * STAGE >= (NW / 2) * NV * 256, "the ring also holds the final reduction");
    extern __shared__ __align__(16) unsigned char smem[];          // NR page buffers, then NW x 64 floats of partial maxima
    float* xchg = reinterpret_cast<float*>(smem + NR * STAGE);

    const int bh = blockIdx.x;
    const int b = bh / Hq, h = bh % Hq;
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pi = wave >> 2, T = (wave >> 1) & 1, t = wave & 1;
    const int q_row = ln;
    const int Hkv = Hq / G;

    // Q operands of row block 0 (rows 0..31 of this head's only tile; rows >= L are zero)
    uint4v qop[KS];
    const size_t grp = (size_t)bh * 4;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = *reinterpret_cast<const uint4v*>(qops + ((grp * KS + ks) * 64 + lane) * 16);
    uint32_t qs = qsc[grp * 64 + lane];

    const int Lk = __builtin_amdgcn_readfirstlane(kv_lens[b]);
    const int koff = Lk - lq_inner;
    const bool packed = lq_inner != L;
    const int nst = min((Lk + 127) / 128, max_pages);              // pages of this sequence
    const int nit = (nst + NP - 1) / NP;
    const int klim = CAUSAL ? min(Lk - 1, koff + (packed ? q_row % lq_inner : q_row)) : Lk - 1;

    // The pages of iteration it: NP * NCH copies of 1 KiB, dealt out to the waves in turn
    auto issue_iter = [&](int it) __attribute__((always_inline)) {
#pragma unroll
        for (int pp = 0; pp < NP; ++pp) {
            const int st = it * NP + pp;
            if (st < nst) {
                int page = __builtin_amdgcn_readfirstlane(page_table[(size_t)b * max_pages + st]);
                page = min(max(page, 0), num_pages - 1);           // a bad table entry reads a wrong page, never outside the cache
                const unsigned char* src = kv + ((size_t)page * Hkv + (h / G)) * STAGE;
                unsigned char* dst = smem + (st % NR) * STAGE;
                // copy g = pp * NCH + ch of the iteration goes to wave g mod NW
                for (int ch = (wave + NW - (pp * NCH) % NW) % NW; ch < NCH; ch += NW)
                    async_copy16(src, (uint32_t)(ch * 1024 + lane * 16), dst + ch * 1024);
            }
        }
    };
    // Wait until all but the copies of the `newer` most recent iterations have landed (vector-memory operations complete
    // in order).  Only meaningful while those iterations are whole: a wave issues (NP * NCH) / NW copies per iteration,
    // the first (NP * NCH) % NW waves one more.  s_waitcnt takes an immediate, hence the branches.
    constexpr int CLO = (NP * NCH) / NW, NHI = (NP * NCH) % NW;
    static_assert(NIT <= 4 && 2 * (CLO + 1) < 16, "at most two newer iterations in flight at a wait; the immediate below has 4 bits");
    auto wait_all_but = [&](int newer) __attribute__((always_inline)) {
#define AQ_VM(N) __builtin_amdgcn_s_waitcnt((N) | 0x70)
        if (newer >= 2)      { if (wave < NHI) AQ_VM(2 * (CLO + 1)); else AQ_VM(2 * CLO); }
        else if (newer == 1) { if (wave < NHI) AQ_VM(CLO + 1); else AQ_VM(CLO); }
        else                 __builtin_amdgcn_s_waitcnt(0);
#undef AQ_VM
    };
    auto as8 = [](const uint4v& x) __attribute__((always_inline)) -> int8v {
        int8v r = {(int)x[0], (int)x[1], (int)x[2], (int)x[3], 0, 0, 0, 0};
        return r;
    };

    floatx16 o[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mt][i] = 0.0f;
    float m_run = -INFINITY;         // maximum after the last iteration (the same in every wave)
    float mref = -INFINITY;          // maximum this wave's O and l refer to (after its tile of its last iteration)
    float lsum = 0.0f;

    // Q must have arrived before the copies start: the wait for an ordinary load issued after them would wait for them too
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qop[ks]));
    asm volatile("" : "+v"(qs));
    __builtin_amdgcn_s_waitcnt(0);
#pragma unroll
    for (int i = 0; i < NIT - 1; ++i)
        if (i < nit) issue_iter(i);

    for (int it = 0; it < nit; ++it) {
        // iteration it's pages are in LDS (the newer ones may be in flight if they are whole), everyone is past iteration it - 1
        const int issued = min(nit, it + NIT - 1);                            // iterations issued so far
        wait_all_but(issued * NP <= nst ? issued - 1 - it : 0);
        __builtin_amdgcn_s_barrier();
        if (it + NIT - 1 < nit) issue_iter(it + NIT - 1);                     // into the buffers of iteration it - 1
        const int st = it * NP + pi;                                          // this wave's page
        const bool valid = st < nst;                                          // (the last iteration may be short of pages)
        const unsigned char* rec = smem + (st % NR) * STAGE + T * REC;
        const int k0 = st * 128 + T * 64;
        // S^T of this wave's 32 keys
        floatx16 sv;
#pragma unroll
        for (int i = 0; i < 16; ++i) sv[i] = -INFINITY;
        if (valid) {
            const uint32_t ksc = lds_read4(rec + KOPS + VOPS + lane * 4);
            uint4v a[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks] = lds_read16(rec + ((t * KS + ks) * 64 + lane) * 16);
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = 0.0f;
            if (t == 0) {
                sv = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0]), as8(qop[0]), sv, 4, 4, 0, ksc, 0, qs);
                if constexpr (KS == 2) sv = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1]), as8(qop[1]), sv, 4, 4, 1, ksc, 1, qs);
            } else {
                sv = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[0]), as8(qop[0]), sv, 4, 4, KS, ksc, 0, qs);
                if constexpr (KS == 2) sv = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(a[1]), as8(qop[1]), sv, 4, 4, 3, ksc, 1, qs);
            }
            const bool need_mask = (k0 + 64 > Lk) || (CAUSAL && k0 + 63 > koff);
            if (need_mask) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (k0 + 32 * hf + 16 * t + i > klim) sv[i] = -INFINITY;
            }
        }
        float pm[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pm[i] = max_nc(max_nc(sv[i], sv[4 + i]), max_raw(sv[8 + i], sv[12 + i]));
        xchg[wave * 64 + lane] = max_nc(max_nc(pm[0], pm[1]), max_nc(pm[2], pm[3]));
        // (fences, not __syncthreads(): the copies in flight are not to be waited for here)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        // maxima after each of the iteration's 2 NP tiles (tile tau: waves 2 tau and 2 tau + 1, both half-waves)
        float mT = m_run, bm = -INFINITY, mt_run = m_run;
#pragma unroll
        for (int tau = 0; tau < 2 * NP; ++tau) {
            const float x0 = xchg[(2 * tau) * 64 + lane], x1 = xchg[(2 * tau + 1) * 64 + lane];
            const float y0 = xchg[(2 * tau) * 64 + (lane ^ 32)], y1 = xchg[(2 * tau + 1) * 64 + (lane ^ 32)];
            mt_run = max_nc(mt_run, max_nc(max_nc(x0, x1), max_nc(y0, y1)));
            if (tau == 2 * pi + T) { mT = mt_run; bm = max_nc(x0, x1); }     // wave-uniform: this wave's tile, this lane's block
        }
        m_run = mt_run;
        if (valid) {
            const float alpha = __builtin_amdgcn_exp2f((mref - mT) * c);
            const float ms = mT * c;
            mref = mT;
            float p[16];
            float rp[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(fmaf(sv[i], c, -ms));
                rp[i & 3] += p[i];
            }
            lsum = lsum * alpha + ((rp[0] + rp[1]) + (rp[2] + rp[3]));        // un-quantized P-tilde
            const float amax = __builtin_amdgcn_exp2f(fmaf(bm, c, -ms));
            const uint32_t pbyte = e8m0_of_amax(amax);
            const float psc = e8m0_as_f32(pbyte);
            uint32_t c0 = 0u, c1 = 0u;
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, p[0], p[1], psc, 0);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, p[2], p[3], psc, 1);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, p[4], p[5], psc, 2);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, p[6], p[7], psc, 3);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, p[8], p[9], psc, 0);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, p[10], p[11], psc, 1);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, p[12], p[13], psc, 2);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, p[14], p[15], psc, 3);
            // B operand of O^T += V^F^T P^T: this lane's k-slots are keys 32 hf + 0..31 of the tile, 8 to a register;
            // the wave fills the 16 it has and leaves the other wave's at zero
            const int8v pb = t ? int8v{0, 0, (int)c0, (int)c1, 0, 0, 0, 0} : int8v{(int)c0, (int)c1, 0, 0, 0, 0, 0, 0};
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[mt][i] *= alpha;
            }
            const uint32_t vsc = lds_read4(rec + KOPS + VOPS + 256 + lane * 4);
            uint4v va[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) va[mt] = lds_read16(rec + KOPS + (mt * 64 + lane) * 16);
            o[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[0]), pb, o[0], 4, 4, 0, vsc, 0, pbyte);
            o[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[1]), pb, o[1], 4, 4, 1, vsc, 0, pbyte);
            if constexpr (MT == 4) {
                o[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[2]), pb, o[2], 4, 4, 2, vsc, 0, pbyte);
                o[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as8(va[3]), pb, o[3], 4, 4, 3, vsc, 0, pbyte);
            }
        }
        // (the partial maxima are read before the next iteration's barrier, which precedes the next writes)
    }

    // ---- the partial results, brought to the final maximum and added (a tree over the waves); O /= l, L = m + log l
    const float f = (mref == m_run) ? 1.0f : __builtin_amdgcn_exp2f((mref - m_run) * c);      // (also covers -inf - -inf)
    float l = xhalf_sum(lsum) * f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mt][i] *= f;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                                                          // everyone is done with the page buffers
    float* red = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int step = NW / 2; step >= 1; step >>= 1) {
        if (wave >= step && wave < 2 * step) {
            float* dst = red + (size_t)(wave - step) * NV * 64;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[(mt * 16 + i) * 64 + lane] = o[mt][i];
            dst[(MT * 16) * 64 + lane] = l;
        }
        __syncthreads();
        if (wave < step) {
            const float* src = red + (size_t)wave * NV * 64;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[mt][i] += src[(mt * 16 + i) * 64 + lane];
            l += src[(MT * 16) * 64 + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
        const float inv_l = l > 0.0f ? 1.0f / l : 0.0f;                       // a sequence without keys: O = 0, L = -inf
        if (q_row < L) {
            const size_t row = (size_t)bh * L + q_row;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    const int d0 = 32 * mt + 8 * tt + 4 * hf;
                    uint2v w;
                    w[0] = pack_bf16x2_rne(o[mt][4 * tt] * inv_l, o[mt][4 * tt + 1] * inv_l);
                    w[1] = pack_bf16x2_rne(o[mt][4 * tt + 2] * inv_l, o[mt][4 * tt + 3] * inv_l);
                    *reinterpret_cast<uint2v*>(O + row * D + d0) = w;
                }
            if (hf == 0) lse[row] = m_run * (c * 0.6931471805599453f) + logf(l);
        }
    }
}

// ---------------------------------------------------------------------------------------------
template <int D>
static int quant_d(const void* x, int BH, int L, int mode, bool fp8v, unsigned char* codes, unsigned char* scales, void* xf,
                   const int* page_ids, int num_pages, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const int rows = mode == 0 ? L : Lp;
    const dim3 grid((unsigned)(((size_t)rows * (D / 32) + 255) / 256), (unsigned)BH);
    if (mode == 0)      hipLaunchKernelGGL((mx_quant_d_kernel<D, 0>), grid, dim3(256), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    else if (mode == 3) hipLaunchKernelGGL((mx_quant_d_kernel<D, 3>), grid, dim3(256), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    else if (mode == 1) hipLaunchKernelGGL((mx_quant_d_kernel<D, 1>), grid, dim3(256), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    else if (fp8v)      hipLaunchKernelGGL((mx_quant_d_kernel<D, 2, true>), grid, dim3(256), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    else                hipLaunchKernelGGL((mx_quant_d_kernel<D, 2>), grid, dim3(256), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
template <int D, bool FP8>
static int quant_l(const void* x, int BH, int L, int mode, unsigned char* codes, unsigned char* scales, void* xf,
                   const int* page_ids, int num_pages, hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const int nblk = mode == 0 ? (L + 31) / 32 : Lp / 32;
    const dim3 grid((unsigned)nblk, (unsigned)BH);
    if (mode == 0) hipLaunchKernelGGL((mx_quant_l_kernel<D, 0, FP8>), grid, dim3(D), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    else           hipLaunchKernelGGL((mx_quant_l_kernel<D, 2, FP8>), grid, dim3(D), 0, st, (const uint16_t*)x, L, Lp, codes, scales, (uint16_t*)xf, page_ids, num_pages);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_mx_quant(const void* x, int BH, int L, int D, int axis, int mode, bool fp8,
                    unsigned char* codes, unsigned char* scales, void* xf, hipStream_t st, const int* page_ids, int num_pages)
{
    if (BH > 65535 || (axis == 0 && fp8 && mode != 2) || (page_ids && (mode != 2 || fp8)) || (mode == 3 && axis != 0)) return -1;
    if (axis == 0) return D == 128 ? quant_d<128>(x, BH, L, mode, fp8, codes, scales, xf, page_ids, num_pages, st) : quant_d<64>(x, BH, L, mode, fp8, codes, scales, xf, page_ids, num_pages, st);
    if (fp8) return D == 128 ? quant_l<128, true>(x, BH, L, mode, codes, scales, xf, page_ids, num_pages, st) : quant_l<64, true>(x, BH, L, mode, codes, scales, xf, page_ids, num_pages, st);
    return D == 128 ? quant_l<128, false>(x, BH, L, mode, codes, scales, xf, page_ids, num_pages, st) : quant_l<64, false>(x, BH, L, mode, codes, scales, xf, page_ids, num_pages, st);
}

size_t mx_kv_bytes(int BHkv, int L, int D, bool fp8v) { return (size_t)BHkv * (round_up(L, kRowPad) / 64) * mx_rec_bytes(D, fp8v); }
size_t mx_ktrain_bytes(int BHkv, int L, int D) { return (size_t)BHkv * (round_up(L, kRowPad) / 64) * mx_ktrain_rec_bytes(D); }
size_t mx_qops_bytes(int BHq, int L, int D) { return (size_t)BHq * round_up(L, kRowPad) * (D / 2); }
size_t mx_qsc_bytes(int BHq, int L) { return (size_t)BHq * (round_up(L, kRowPad) / 32) * 64 * 4; }
size_t mx_page_bytes(int D) { return 2 * (size_t)mx_rec_bytes(D, false); }

template <int D, bool CAUSAL, bool FP8PV, int KVM>
static int launch_fwd_mx_t(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L,
                           void* o, float* lse, const int* page_table, const int* kv_lens, int max_pages, int num_pages, int lq_inner,
                           hipStream_t st)
{
    const int Lp = round_up(L, kRowPad);
    const size_t smem = 3 * 2 * (size_t)mx_rec_bytes(D, FP8PV);
    auto kern = fwd_mx_kernel<D, CAUSAL, FP8PV, KVM>;
    static unsigned long long lds_set = 0;          // one per instantiation
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return -1;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq * (Lp / 128))), dim3(256), smem, st,
                       (const unsigned char*)qops, (const uint32_t*)qsc, (const unsigned char*)kv,
                       (uint16_t*)o, lse, L, Lp, Hq, Hq / Hkv, c, page_table, kv_lens, max_pages, num_pages, lq_inner);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
template <int D, bool FP8PV>
static int launch_fwd_mx_d(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L, bool causal,
                           void* o, float* lse, hipStream_t st)
{
    return causal ? launch_fwd_mx_t<D, true, FP8PV, 0>(qops, qsc, kv, B, Hq, Hkv, L, o, lse, nullptr, nullptr, 0, 0, L, st)
                  : launch_fwd_mx_t<D, false, FP8PV, 0>(qops, qsc, kv, B, Hq, Hkv, L, o, lse, nullptr, nullptr, 0, 0, L, st);
}

int launch_fwd_mx(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L, int D, bool causal, bool fp8pv,
                  void* o, float* lse, hipStream_t st)
{
    if (D == 128) return fp8pv ? launch_fwd_mx_d<128, true>(qops, qsc, kv, B, Hq, Hkv, L, causal, o, lse, st)
                               : launch_fwd_mx_d<128, false>(qops, qsc, kv, B, Hq, Hkv, L, causal, o, lse, st);
    if (D == 64)  return fp8pv ? launch_fwd_mx_d<64, true>(qops, qsc, kv, B, Hq, Hkv, L, causal, o, lse, st)
                               : launch_fwd_mx_d<64, false>(qops, qsc, kv, B, Hq, Hkv, L, causal, o, lse, st);
    return -1;
}

int launch_fwd_mx_paged(const void* qops, const void* qsc, const void* cache, int B, int Hq, int Hkv, int Lq, int D, bool causal,
                        const int* page_table, const int* kv_lens, int max_pages, int num_pages, int lq_inner,
                        void* o, float* lse, hipStream_t st)
{
    if (Lq <= 32) {
        // a step of decoding: the four waves of a workgroup share the keys of a page
        const float c = 1.4426950408889634f / sqrtf((float)D);
#define AQ_DECODE(DD, CC) do { \
        constexpr int NP = AQ_DECODE_NP; \
        constexpr size_t smem = (NP == 1 ? 4 : NP == 2 ? 3 : 2) * NP * 2 * (size_t)mx_rec_bytes(DD, false) + 4 * NP * 256; \
        auto kern = fwd_mx_decode_kernel<DD, CC, NP>; \
        static unsigned long long lds_set = 0; \
        if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return -1; \
        hipLaunchKernelGGL(kern, dim3((unsigned)(B * Hq)), dim3(256 * NP), smem, st, (const unsigned char*)qops, (const uint32_t*)qsc, \
                           (const unsigned char*)cache, (uint16_t*)o, lse, Lq, Hq, Hq / Hkv, c, page_table, kv_lens, max_pages, num_pages, lq_inner); \
        return hipGetLastError() == hipSuccess ? 0 : -1; } while (0)
        if (D == 128) { if (causal) AQ_DECODE(128, true); else AQ_DECODE(128, false); }
        if (D == 64)  { if (causal) AQ_DECODE(64, true); else AQ_DECODE(64, false); }
#undef AQ_DECODE
        return -1;
    }
#define AQ_PAGED(DD, CC) launch_fwd_mx_t<DD, CC, false, 1>(qops, qsc, cache, B, Hq, Hkv, Lq, o, lse, page_table, kv_lens, max_pages, num_pages, lq_inner, st)
    if (D == 128) return causal ? AQ_PAGED(128, true) : AQ_PAGED(128, false);
    if (D == 64)  return causal ? AQ_PAGED(64, true) : AQ_PAGED(64, false);
#undef AQ_PAGED
    return -1;
}

// Block lists of the block-sparse forward: row r = (b * Hq + h) * nqb + query block of mask [rows, nkb] (bytes, zero =
// the block is left out) -> the indices of its non-zero key blocks in increasing order, and their number.
__global__ void mx_block_list_kernel(const unsigned char* __restrict__ mask, int nrows, int nkb, int* __restrict__ list, int* __restrict__ cnt)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= nrows) return;
    int n = 0;
    for (int kb = 0; kb < nkb; ++kb)
        if (mask[(size_t)r * nkb + kb]) list[(size_t)r * nkb + n++] = kb;
    cnt[r] = n;
}

int launch_fwd_mx_sparse(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L, int D, bool causal,
                         const unsigned char* block_mask, int* list, int* cnt, void* o, float* lse, hipStream_t st)
{
    const int nb = round_up(L, kRowPad) / 128, nrows = B * Hq * nb;
    hipLaunchKernelGGL(mx_block_list_kernel, dim3((unsigned)((nrows + 127) / 128)), dim3(128), 0, st, block_mask, nrows, nb, list, cnt);
    if (hipGetLastError() != hipSuccess) return -1;
#define AQ_SPARSE(DD, CC) launch_fwd_mx_t<DD, CC, false, 2>(qops, qsc, kv, B, Hq, Hkv, L, o, lse, list, cnt, nb, 0, L, st)
    if (D == 128) return causal ? AQ_SPARSE(128, true) : AQ_SPARSE(128, false);
    if (D == 64)  return causal ? AQ_SPARSE(64, true) : AQ_SPARSE(64, false);
#undef AQ_SPARSE
    return -1;
}

}  // namespace aq
