// Host-side launchers of the gfx950 kernels (one translation unit each).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aq {

// phi (+ layout copies).  x [BH, L, D] bf16.  Any output may be null.
//   codes/scales/xf_pub: the public packed NVFP4 tensor and its bf16 dequantized copy
//   xr [BH, Lp, D]: dequantized rows, zero padded to Lp = round_up(L, 128)
//   xt [BH, D, Lp]: the same, transposed, sequence positions permuted inside groups of 16
//   quant=false copies x unchanged (bf16 only).  out_f16 selects fp16 for xr/xt.
//   sub (optional) [BH, D] fp32: subtracted from every row before phi (K smoothing: the token mean of each channel)
int launch_prep(const void* x, int BH, int L, int D, bool quant, bool out_f16,
                uint8_t* codes, uint8_t* scales, void* xf_pub, void* xr, void* xt, hipStream_t st,
                const float* sub = nullptr);

// The layout copies xr / xt (as launch_prep writes them) from an already quantized tensor: codes [BH, L, D/2] and E4M3
// scale bytes [BH, L, D/16] in the layout attnqat_quantize produces.
int launch_unpack(const uint8_t* codes, const uint8_t* scales, int BH, int L, int D, bool out_f16, void* xr, void* xt, hipStream_t st);

// Token mean of every channel of x [BH, L, D] bf16 -> mean [BH, D] fp32 (fp64 sums in a fixed order).
// scratch: colmean_scratch_bytes() bytes.
size_t colmean_scratch_bytes(int BH, int D);
int launch_colmean(const void* x, int BH, int L, int D, double* scratch, float* mean, hipStream_t st);

// Alg. 1 (train=false) / Alg. 2 (train=true) on fp16 copies made by launch_prep.
// p_quant 1 (MX): qh and kh are NOT fp16 copies but the operand arrays of the scaled FP4 instruction (launch_mx_quant mode 1
// for Q, with its scale dwords in qsc, and mode 3 for K): the scores are computed from the codes; vt stays the fp16 copy.
// p_quant: phi(P-tilde) 0 NVFP4; 1 in the MX format (blocks of 32 keys, power-of-two scale); 2 NVFP4 after the
// two-level row factor (every 64-key tile row divided by a power of two that brings its maximum just below 448 * 6).
int launch_fwd(const void* qh, const void* kh, const void* vt,
               int B, int Hq, int Hkv, int L, int D, bool causal, bool train, int p_quant,
               void* o, float* lse, float* o_hp, int dump_row0, float* p_dump, hipStream_t st, const void* qsc = nullptr);

// Alg. 1 for sequences of different lengths (serving): queries are the last Lq positions of every sequence, sequence b has
// kv_lens[b] keys (device array), kh / vt are laid out for Lkp positions per kv head.
int launch_fwd_varlen(const void* qh, const void* kh, const void* vt, int B, int Hq, int Hkv, int Lq, int Lkp, int D, bool causal,
                      const int* kv_lens, void* o, float* lse, hipStream_t st);

// The NVFP4 KV cache (pages of 128 positions; per kv head K codes, K scales, V codes, V scales in the public layout).
size_t nvfp4_page_bytes(int Hkv, int D);
int launch_kv_page_write(const void* k, const void* v, int Hkv, int n, int D, int pos0,
                         void* cache, int num_pages, const int* page_ids, hipStream_t st);
// which: 0 the K part (xr: rows), 1 the V part (xt: transposed); copies laid out for max_pages * 128 positions per sequence
int launch_unpack_pages(const void* cache, const int* page_table, const int* kv_lens, int B, int Hkv, int max_pages, int num_pages,
                        int D, int which, void* xr, void* xt, hipStream_t st);

// Alg. 1 for decode steps over the NVFP4 pages: at most decode_max_rows() query rows per (sequence, kv head), i.e.
// (Hq / Hkv) * Lq of them; qh [B*Hkv][128][D] fp16 is phi(Q) with the rows of a kv group together (launch_prep on q taken as
// [B*Hkv, (Hq/Hkv)*Lq, D]).  ws: decode_ws_bytes() bytes.  spin_limit bounds the polls of a chunk waiting for the row maxima
// of the chunks before it (see decode.hip); if it runs out the int at ws + 4 is set and that result is wrong.
int decode_max_rows();
int decode_chunk_keys(int R);
size_t decode_ws_bytes(int B, int Hkv, int R, int max_pages, int D);
int launch_decode(const void* qh, const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                  int B, int Hq, int Hkv, int Lq, int D, bool causal, void* ws, int spin_limit, void* o, float* lse, hipStream_t st);

// The MX format's operand arrays of the scaled FP4 instruction, from which the backward recomputes the scores (launch_mx_quant):
// qops / qsc: mode 1 on Q; kops / ksc: mode 1 on K (a wave's 32 keys as the A operand of the dK/dV pass); krec: mode 3 on K
// (64-key records, the A operand of the dQ pass).
struct MxScoreOps { const void *qops, *qsc, *kops, *ksc, *krec; };

// Per-row statistics of the backward: rowstat [BHq, Lp, 2] = {L log2(e), D / sqrt(d)} with
// D = rowsum(dO o O') (Alg. 3, first line); padding rows hold zeros.  d_o bf16, o_hp fp32, [rows, D].
// o_acc: O' fp32, or (ablation) the bf16 O when o_is_bf16.
int launch_delta(const void* d_o, const void* o_acc, bool o_is_bf16, const float* lse, int BHq, int L, int D,
                 float* rowstat, hipStream_t st);

// Per-head bounds that limit |dS| (partial maxima of |V^F_j|, |dO_i|, |D_i|/sqrt(d)): part holds
// 3 * BHq * 64 floats.  vb, dob: bf16 row-major copies padded to Lp rows.
int launch_bounds(const void* vb, const void* dob, const float* rowstat, int BHkv, int BHq, int L, int D,
                  float* part, hipStream_t st);

// Alg. 3, query-stationary pass: dQ.  qh, kh: fp16 copies; vb, dob: bf16 copies.
int launch_bwd_dq(const void* qb, const void* kb, const void* vb, const void* dob,
                  const float* rowstat, const float* bound_part,
                  int B, int Hq, int Hkv, int L, int D, bool causal, void* dq, hipStream_t st,
                  const MxScoreOps* mx = nullptr /* the MX format: scores from the codes */);

// Alg. 3, key-stationary pass: dK, dV (summed over the query heads of a group).
int launch_bwd_dkdv(const void* qb, const void* kb, const void* vb, const void* dob,
                    const float* rowstat, const float* bound_part,
                    int B, int Hq, int Hkv, int L, int D, bool causal, void* dk, void* dv,
                    unsigned long long* tile_counts /* may be null */,
                    int p_quant /* phi(P): 0 none (ablation), 1 NVFP4, 2 MX, 3 NVFP4 with the two-level row factor */, hipStream_t st,
                    float* p_dump = nullptr /* test hook, p_quant 1 only: P^F of query rows [dump_row0, dump_row0 + 128), [B*Hq][128][L] */,
                    int dump_row0 = 0, const MxScoreOps* mx = nullptr /* p_quant 2: required */);
// Waves per workgroup of the dQ and dK/dV passes: 0 = chosen per problem (the default), 4 or 8 = forced where that
// variant exists (8: not the ablation and not the counting variant).  Process-wide; for tests.
void set_bwd_waves(int waves);

// ---- MX variant (E2M1, blocks of 32, E8M0 scale; mx.hip) ----
// phi with the blocks along d (axis 0) or along the sequence (axis 1).  x [BH, L, D] bf16.
//   mode 0: public layout (codes, scales, optional bf16 xf, see attnqat.h)
//   mode 1: Q operands of the scaled MFMA (axis 0 only): codes -> operand array, scales -> scale dwords
//   mode 2: the K part (axis 0) or the V part (axis 1) of the 64-key kv records at `codes`
//   mode 3: K records of the training forward (axis 0 only): natural key order, see mx.hip
// fp8: E4M3 elements instead of E2M1 (axis 1 only); with axis 0 and mode 2 it selects the record layout whose V part is FP8.
// page_ids (mode 2, FP4 only; device int32, one entry per 128 positions): the records go into the pages of a KV cache
// laid out [page][kv head][2 records] instead of one after another; BH then is the number of kv heads of ONE sequence.
// Records whose page id lies outside [0, num_pages) are not written.
int launch_mx_quant(const void* x, int BH, int L, int D, int axis, int mode, bool fp8,
                    unsigned char* codes, unsigned char* scales, void* xf, hipStream_t st, const int* page_ids = nullptr, int num_pages = 0);
size_t mx_kv_bytes(int BHkv, int L, int D, bool fp8v);
size_t mx_ktrain_bytes(int BHkv, int L, int D);      // K records of the MX training forward (launch_mx_quant mode 3)
size_t mx_qops_bytes(int BHq, int L, int D);
size_t mx_qsc_bytes(int BHq, int L);
// Alg. 1 on the arrays made by launch_mx_quant (modes 1 and 2).  fp8pv: P-tilde and V in MXFP8 (mixed recipe).
int launch_fwd_mx(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L, int D, bool causal, bool fp8pv,
                  void* o, float* lse, hipStream_t st);

// The same forward on a paged KV cache: a head has Lq rows, positions kv_lens[b] - lq_inner .. of its sequence, repeated
// Lq / lq_inner times when the query heads of a kv group are packed into one head (then Hq == Hkv).
size_t mx_page_bytes(int D);
int launch_fwd_mx_paged(const void* qops, const void* qsc, const void* cache, int B, int Hq, int Hkv, int Lq, int D, bool causal,
                        const int* page_table, const int* kv_lens, int max_pages, int num_pages, int lq_inner,
                        void* o, float* lse, hipStream_t st);

// Block-sparse forward on contiguous kv records: block_mask [B*Hq*nb, nb] bytes with nb = ceil(L/128); list
// ([B*Hq*nb, nb] int32) and cnt ([B*Hq*nb] int32) are scratch that the call fills.
int launch_fwd_mx_sparse(const void* qops, const void* qsc, const void* kv, int B, int Hq, int Hkv, int L, int D, bool causal,
                         const unsigned char* block_mask, int* list, int* cnt, void* o, float* lse, hipStream_t st);

}  // namespace aq
