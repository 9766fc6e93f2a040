/*
 * attnqat.h -- C ABI of the MI355X (gfx950) Attn-QAT hot path.
 *
 * NVFP4 fake-quantized attention: E2M1 elements with one E4M3 scale per 16
 * elements (Sec. 2.1, Eq. 1-2), the inference forward (Alg. 1), the training
 * forward that also emits the high-precision output O' (Alg. 2) and the
 * backward that re-quantizes the recomputed P and takes D from O' (Alg. 3).
 *
 * Beyond that core (each group is described where it is declared):
 *   attnqat_bwd_ablation                the two backward ablations of Sec. 3.2
 *   attnqat_fwd_opt, attnqat_bwd_opt    K smoothing and two-level quantization of P (Sec. 2.1 / 4.2) as option bits
 *   attnqat_quantize_mx, attnqat_fwd_infer_mx, attnqat_fwd_mx, attnqat_bwd_mx
 *                                       the same method in the MX format (E2M1 blocks of 32, E8M0 scales), whose
 *                                       inference forward runs on the scaled FP4 matrix instruction
 *   attnqat_quantize_mxfp8, attnqat_fwd_infer_mx_fp8pv   the mixed recipe: FP4 Q K^T, FP8 P V
 *   attnqat_kv_cache_*, attnqat_fwd_infer_mx_paged       an FP4 KV cache in pages and the forward over it
 *   attnqat_fwd_infer_mx_sparse                          block-sparse attention
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a caller-owned DEVICE pointer (HBM).  Nothing is
 *     allocated, freed or synchronised here: kernels are enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns.  Scratch memory comes in through `workspace`; ask
 *     attnqat_workspace_bytes() for its size.  The workspace may be reused by
 *     the next call on the same stream.
 *   - Tensors are contiguous, [B, H, L, d] with d innermost.  q/o/d_o/dq/o_hp
 *     have H = Hq heads; k/v/dk/dv have H = Hkv heads; Hq % Hkv == 0 and query
 *     head h reads kv head h / (Hq/Hkv) (grouped-query attention).
 *   - L is both the query and the key length (except in attnqat_fwd_infer_mx_paged).  d is 64 or 128.
 *   - dtype: ATTNQAT_BF16 (the only supported storage type of q,k,v,d_o and
 *     of o,dq,dk,dv).  lse is fp32, o_hp is fp32.
 *   - causal != 0: query i sees keys 0..i.
 *   - Return value: ATTNQAT_OK or a negative ATTNQAT_E* code; on error no
 *     kernel has been enqueued.  attnqat_strerror() names a code.
 *   - P is quantized in groups of 16 consecutive keys aligned to absolute key
 *     indices that are multiples of 16; key tiles of attnqat_block_k() keys are
 *     visited in increasing order and P-tilde of a tile is quantized against
 *     the running row maximum after that tile (Alg. 1/2 inner loop).  The key
 *     tile size therefore is part of the forward's definition.
 */
#ifndef ATTNQAT_H
#define ATTNQAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ATTNQAT_OK                  0
#define ATTNQAT_EINVAL             -1   /* null pointer, non-positive size            */
#define ATTNQAT_ESHAPE             -2   /* d not in {64,128}, Hq % Hkv != 0, L too big */
#define ATTNQAT_EDTYPE             -3   /* dtype other than ATTNQAT_BF16              */
#define ATTNQAT_EWORKSPACE         -4   /* workspace null or smaller than required    */
#define ATTNQAT_ELAUNCH            -5   /* the HIP runtime refused a launch           */
#define ATTNQAT_ESTATIC            -6   /* attnqat_fwd_infer_static: needs more than ATTNQAT_STATIC_SCRATCH_BYTES */

#define ATTNQAT_BF16                0

#define ATTNQAT_WS_FWD              0   /* attnqat_fwd                                 */
#define ATTNQAT_WS_FWD_INFER        1   /* attnqat_fwd_infer                           */
#define ATTNQAT_WS_BWD              2   /* attnqat_bwd                                 */
#define ATTNQAT_WS_FWD_INFER_MX     3   /* attnqat_fwd_infer_mx                        */
#define ATTNQAT_WS_FWD_MX           4   /* attnqat_fwd_mx, attnqat_debug_fwd_p_mx      */
#define ATTNQAT_WS_BWD_MX           5   /* attnqat_bwd_mx                              */
#define ATTNQAT_WS_FWD_INFER_MX_FP8PV 6 /* attnqat_fwd_infer_mx_fp8pv                  */
#define ATTNQAT_WS_FWD_INFER_MX_PAGED 7 /* attnqat_fwd_infer_mx_paged (L = queries per sequence) */
#define ATTNQAT_WS_FWD_INFER_MX_SPARSE 8 /* attnqat_fwd_infer_mx_sparse                        */

/*
 * phi of Eq. 1 (Sec. 2.1) along d: for every 16 consecutive elements
 *   scale = RNE_E4M3(max|x| / 6)   (saturating at 448; a scale of 0 zeroes the block)
 *   code  = sign | RNE_E2M1(|x| / scale)   (ties to even, saturating at 6)
 * x       [B,H,L,d] bf16 (device, read)
 * codes   [B,H,L,d/2] bytes (device, written): element 2k in bits 3:0, 2k+1 in bits 7:4;
 *         a code is sign<<3 | index into {0,.5,1,1.5,2,3,4,6}
 * scales  [B,H,L,d/16] E4M3 bytes (device, written)
 * xf      optional [B,H,L,d] bf16 (device, written): phi^-1(phi(x)) of Eq. 2; may be NULL
 * codes and scales may be NULL when only xf is wanted.  Alignment (vector loads and stores): x and xf 16 bytes, codes 8,
 * scales 4; otherwise ATTNQAT_EINVAL.
 */
int attnqat_quantize(const void* x, int B, int H, int L, int d, int dtype,
                     uint8_t* codes, uint8_t* scales, void* xf, void* stream);

/*
 * Training forward, Alg. 2: fake-quantizes q, k, v, runs the online-softmax
 * recurrence with P-tilde fake-quantized before P.V, and also accumulates
 * O' = sum P-tilde V^F with the un-quantized P-tilde.
 * q [B,Hq,L,d], k,v [B,Hkv,L,d] bf16 (read)
 * o    [B,Hq,L,d] bf16 (written)      lse [B,Hq,L] fp32 (written, natural log)
 * o_hp [B,Hq,L,d] fp32 (written): O', for attnqat_bwd only
 */
int attnqat_fwd(const void* q, const void* k, const void* v,
                int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                void* o, float* lse, float* o_hp,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Inference forward, Alg. 1 (the same O and lse as attnqat_fwd by Eq. 3 == Eq. 4,
 * without O').  The Q/K/V quantization pass is part of the call.
 */
int attnqat_fwd_infer(const void* q, const void* k, const void* v,
                      int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                      void* o, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * The packed-input forms: Alg. 1 as the paper writes it takes the quantized tensors (Q-hat, s_Q, K-hat, s_K, V-hat, s_V),
 * and its training setup (appendix "Detailed Training Setup") saves the fake-quantized Q, K, V of the forward for the
 * backward.  *_codes [B,H,L,d/2] and *_scales [B,H,L,d/16] are what attnqat_quantize wrote for q, k, v (H = Hq for q,
 * Hkv for k and v; codes 8-byte aligned); everything else is as in attnqat_fwd_infer / attnqat_bwd, including the
 * workspace sizes (ATTNQAT_WS_FWD_INFER, ATTNQAT_WS_BWD), and the results are bit-identical to those calls on the
 * tensors the codes came from: the quantization pass is replaced by a pass that only unpacks (0.56 instead of 2 bytes
 * read per element).  dtype is the type of o, d_o, dq, dk, dv (ATTNQAT_BF16).
 */
int attnqat_fwd_infer_packed(const uint8_t* q_codes, const uint8_t* q_scales, const uint8_t* k_codes, const uint8_t* k_scales,
                             const uint8_t* v_codes, const uint8_t* v_scales,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);
int attnqat_bwd_packed(const uint8_t* q_codes, const uint8_t* q_scales, const uint8_t* k_codes, const uint8_t* k_scales,
                       const uint8_t* v_codes, const uint8_t* v_scales, const void* d_o,
                       const float* lse, const float* o_hp,
                       int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                       void* dq, void* dk, void* dv,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * attnqat_fwd_infer for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit for bit)
 * as attnqat_fwd_infer, without the workspace: the scratch memory is a fixed array of ATTNQAT_STATIC_SCRATCH_BYTES
 * inside the library's device image, which every GPU that the library runs on holds until the process ends.
 *   - Problems with attnqat_workspace_bytes(ATTNQAT_WS_FWD_INFER, ...) > ATTNQAT_STATIC_SCRATCH_BYTES are refused with
 *     ATTNQAT_ESTATIC and nothing is enqueued (e.g. B=1, Hq=8, Hkv=2, L=8192, d=128 needs 24.1 MiB and fits).
 *   - Calls nothing that allocates or frees.  The first call on a device looks up the array's device address
 *     (hipGetSymbolAddress, once per device, kept); make that first call outside a graph capture.
 *   - All calls on one GPU share the one array: calls that may overlap on a GPU (different streams, different
 *     threads) race on it.  Calls on one stream are ordered and safe.  Nothing needs clearing between calls: the
 *     quantization pass rewrites every byte the forward reads.
 */
#define ATTNQAT_STATIC_SCRATCH_BYTES (32u << 20)
int attnqat_fwd_infer_static(const void* q, const void* k, const void* v,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* stream);

/*
 * Backward, Alg. 3, with straight-through estimation (Eq. 5):
 *   D = rowsum(dO o O');  P = exp(S - lse);  P^F = phi^-1(phi(P));
 *   dV = P^F^T dO;  dP = dO V^F^T;  dS = P o (dP - D)/sqrt(d);  dQ = dS K^F;  dK = dS^T Q^F.
 * q,k,v are the un-quantized inputs of the forward (they are fake-quantized
 * again here, which is bit-identical); d_o [B,Hq,L,d] bf16; lse and o_hp are
 * the forward's outputs.  dq [B,Hq,L,d], dk,dv [B,Hkv,L,d] bf16 (written; dk and
 * dv are summed over the Hq/Hkv query heads of a group).
 */
int attnqat_bwd(const void* q, const void* k, const void* v, const void* d_o,
                const float* lse, const float* o_hp,
                int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                void* dq, void* dk, void* dv,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two backward ablations of Sec. 3.2 (Table 2, Exp. 7 and Exp. 8; the failure modes that
 * Sec. 2.3 explains), as switches of the same backward.  `ablation` is a bit set:
 *   ATTNQAT_ABL_D_FROM_O       D = rowsum(dO o O) with the forward's low-precision output `o`
 *                              ([B,Hq,L,d] bf16, device, read) instead of O'; o_hp is ignored.
 *   ATTNQAT_ABL_P_UNQUANTIZED  dV += P^T dO with the recomputed fp32 P instead of
 *                              phi^-1(phi(P)) (P enters the product as a bf16 hi + lo pair).
 * 0 computes exactly what attnqat_bwd computes.  Other arguments, workspace, errors: as attnqat_bwd
 * (workspace size ATTNQAT_WS_BWD); `o` may be NULL unless ATTNQAT_ABL_D_FROM_O is set, o_hp may be
 * NULL if it is.
 */
#define ATTNQAT_ABL_D_FROM_O        1
#define ATTNQAT_ABL_P_UNQUANTIZED   2
int attnqat_bwd_ablation(const void* q, const void* k, const void* v, const void* d_o,
                         const float* lse, const float* o_hp, const void* o,
                         int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int ablation,
                         void* dq, void* dk, void* dv,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace the call named by `which` (ATTNQAT_WS_*) needs; 0 for bad arguments. */
size_t attnqat_workspace_bytes(int which, int B, int Hq, int Hkv, int L, int d);

/* The key tile size B_k of Alg. 1/2 that the forward kernels implement. */
int attnqat_block_k(void);

/* Static, NUL-terminated description of a return code. */
const char* attnqat_strerror(int code);

/*
 * Test hook: attnqat_fwd_infer that also writes the dequantized P-tilde^F that
 * entered the O update, for the 128 query rows [row0, row0+128) of every head
 * (row0 a multiple of 128): p_dump [B,Hq,128,L] fp32 (device).  The caller
 * zeroes it before the call (none of the three P hooks clears it): key tiles
 * that no row of a 32-row group can see under the causal mask are skipped and
 * not written, nor are rows beyond L; masked keys inside a visited tile get 0.
 */
int attnqat_debug_fwd_p(const void* q, const void* k, const void* v,
                        int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                        void* o, float* lse, int row0, float* p_dump,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Test hook: attnqat_bwd that also writes P^F = phi^-1(phi(P)), the re-quantized recomputed P that enters
 * dV = P^F^T dO (Alg. 3), for the 128 query rows [row0, row0+128) of every head and all keys: p_dump [B,Hq,128,L] fp32
 * (device).  The caller zeroes it before the call: tiles of 32 queries x 32 keys in which every block scale rounds to 0
 * are skipped (their P^F is 0) and not written, nor are masked keys and rows beyond L.
 */
int attnqat_debug_bwd_p(const void* q, const void* k, const void* v, const void* d_o,
                        const float* lse, const float* o_hp,
                        int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                        void* dq, void* dk, void* dv, int row0, float* p_dump,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * The NVFP4 forward and backward with options that Sec. 3.2 studies inside QAT (SageAttention's heuristics):
 *   ATTNQAT_OPT_SMOOTH_K   K smoothing (Sec. 2.1): phi is applied to K minus its mean over the tokens, per
 *                          (batch, kv head, channel).  S changes by a per-query constant that softmax ignores
 *                          (lse moves by q . mean(K) / sqrt(d)); the centred K quantizes better.  The mean is the
 *                          fp64 sum / L rounded to fp32, the subtraction an fp32 subtraction.  dK is the gradient
 *                          with respect to the centred K, which equals the gradient with respect to K because
 *                          rowsum(dS) = 0 when D comes from O' (Sec. 2.3).
 *   ATTNQAT_OPT_TWO_LEVEL_P  two-level quantization of P (Sec. 2.1): every row of a 64-key tile of P-tilde (forward)
 *                          and every row of the same aligned groups of 64 keys (key indices 64 g .. 64 g + 63) of the
 *                          recomputed P (backward) is divided by s1, the smallest power of two with
 *                          448 * 6 * s1 >= max(maximum of the row over those 64 keys, 2^-24), quantized in NVFP4
 *                          blocks of 16 and multiplied back, so that blocks far below the row maximum of the whole
 *                          sequence keep their values instead of under-flowing the E4M3 scale.  Masked keys and keys
 *                          beyond L count as 0.  Only P^F changes (O, dV).
 *   ATTNQAT_OPT_BF16_PV    the mixed recipe that Sec. 2.5 proposes against the cost of quantizing P in the kernel:
 *                          S = Q^F K^F^T on NVFP4 operands as everywhere, but P-tilde is only rounded to bf16 (nearest
 *                          even) and V is used as given (bf16, not quantized), so the P V product is a bf16 product with
 *                          fp32 accumulation.  m, l and lse are untouched.  Inference forward only (o_hp must be NULL;
 *                          attnqat_bwd_opt refuses the bit); not together with ATTNQAT_OPT_TWO_LEVEL_P (P has no blocks
 *                          here): ATTNQAT_EINVAL.  attnqat_fwd_infer_bf16pv is attnqat_fwd_opt with this bit alone.
 * attnqat_fwd_opt: o_hp != NULL selects the training forward (Alg. 2), NULL the inference forward (Alg. 1).
 * attnqat_bwd_opt must be given the same options as the forward whose lse and o_hp it consumes.
 * options = 0 is attnqat_fwd / attnqat_fwd_infer / attnqat_bwd; unknown bits: ATTNQAT_EINVAL.
 * Workspace sizes: ATTNQAT_WS_FWD and ATTNQAT_WS_BWD.
 */
#define ATTNQAT_OPT_SMOOTH_K        1
#define ATTNQAT_OPT_TWO_LEVEL_P     2
#define ATTNQAT_OPT_BF16_PV         4
int attnqat_fwd_opt(const void* q, const void* k, const void* v,
                    int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                    void* o, float* lse, float* o_hp,
                    void* workspace, size_t workspace_bytes, void* stream);
int attnqat_bwd_opt(const void* q, const void* k, const void* v, const void* d_o,
                    const float* lse, const float* o_hp,
                    int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                    void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes, void* stream);

int attnqat_fwd_infer_bf16pv(const void* q, const void* k, const void* v,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* attnqat_debug_fwd_p with the option bits of attnqat_fwd_opt (workspace ATTNQAT_WS_FWD). */
int attnqat_debug_fwd_p_opt(const void* q, const void* k, const void* v,
                            int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                            void* o, float* lse, int row0, float* p_dump,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * MX variant of phi: the OCP microscaling FP4 format that Sec. 2.1 names beside NVFP4
 * (E2M1 elements, 32 per block, one power-of-two E8M0 scale), with the power-of-two
 * counterpart of Eq. 1 as the scale rule:
 *   scale = the smallest 2^e, e >= -126, with 6 * 2^e >= max|x|   (byte e + 127; no element saturates)
 *   code  = sign | RNE_E2M1(|x| / scale)
 * axis 0: blocks of 32 along d (how Q and K are blocked)
 *   codes [B,H,L,d/2] bytes (element 2k in bits 3:0), scales [B,H,L,d/32] E8M0 bytes
 * axis 1: blocks of 32 along the sequence, aligned to multiples of 32 and zero padded (how V is
 *   blocked, so that P.V contracts over the blocked axis); with Lc = L rounded up to 32
 *   codes [B,H,d,Lc/2] bytes (position 2k in bits 3:0), scales [B,H,d,Lc/32] E8M0 bytes
 * x [B,H,L,d] bf16 (device, read); xf optional [B,H,L,d] bf16: phi^-1(phi(x)); any output may be
 * NULL, not all three.
 */
int attnqat_quantize_mx(const void* x, int B, int H, int L, int d, int dtype, int axis,
                        uint8_t* codes, uint8_t* scales, void* xf, void* stream);

/*
 * Inference forward, Alg. 1, in the MX format: Q^F, K^F blocked along d, V^F and P-tilde^F along
 * the keys (P blocks of 32 keys aligned to multiples of 32; key tiles of attnqat_block_k() keys
 * as in attnqat_fwd_infer).  Both products run on the scaled FP4 matrix instruction of gfx950 on
 * the codes and scale bytes themselves (Eq. 3: FP4MM), nothing is dequantized.
 * Arguments as attnqat_fwd_infer; workspace size: ATTNQAT_WS_FWD_INFER_MX.
 */
int attnqat_fwd_infer_mx(const void* q, const void* k, const void* v,
                         int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                         void* o, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Mixed recipe of Sec. 2.5 (FP4 for Q K^T, FP8 for P V) in MX terms: Q^F, K^F as in attnqat_fwd_infer_mx;
 * V^F and P-tilde^F in MXFP8: E4M3 elements (OCP: bias 7, subnormals, largest value 448), the same blocks
 * of 32 keys and E8M0 scales, scale = the smallest 2^e, e >= -126, with 448 * 2^e >= max|x| (nothing
 * saturates), element = sign | RNE_E4M3(|x| / scale).  P.V runs on the same scaled matrix instruction with
 * FP8 operands, at half the FP4 rate.  Arguments as attnqat_fwd_infer; workspace ATTNQAT_WS_FWD_INFER_MX_FP8PV.
 *
 * attnqat_quantize_mxfp8: that quantizer for a whole tensor, blocks along the sequence only (axis must be 1):
 *   codes [B,H,d,Lc] E4M3 bytes (Lc = L rounded up to 32, zero padded), scales [B,H,d,Lc/32] E8M0 bytes,
 *   xf optional [B,H,L,d] bf16 (values with more than 8 significant bits are rounded to bf16).
 */
int attnqat_quantize_mxfp8(const void* x, int B, int H, int L, int d, int dtype, int axis,
                           uint8_t* codes, uint8_t* scales, void* xf, void* stream);
int attnqat_fwd_infer_mx_fp8pv(const void* q, const void* k, const void* v,
                               int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                               void* o, float* lse,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Serving: an FP4 KV cache in pages, and Alg. 1 over it for sequences of different lengths (the variable-length /
 * paged setting that Sec. 5 leaves as future work; format and forward as attnqat_fwd_infer_mx).
 *
 * The cache is caller-owned device memory of num_pages * attnqat_kv_cache_page_bytes(Hkv, d) bytes.  A page holds
 * 128 consecutive positions of ONE sequence for all Hkv heads, as MX codes and scale bytes in the order the matrix
 * instruction reads them (K blocked along d, V in blocks of 32 positions), so the scale factors travel with their
 * page and a page table is all a reader needs.
 *
 * attnqat_kv_cache_write_mx quantizes k, v [1,Hkv,L,d] bf16 (positions 0..L-1 of one sequence, L >= 1) into the pages
 * page_ids[0 .. ceil(L/128)-1] (device int32) of a cache of num_pages pages; a last page that is not full is zero
 * padded.  A page id outside [0, num_pages) is not written at all (the ids live on the device, so the call cannot
 * refuse them; nothing outside the cache is touched).  A sequence that grows is written again from position 0 of its
 * last page on (V scales cover 32 positions: a block that gains positions must be re-quantized), i.e. k, v must start
 * at a multiple of 128 of the sequence.
 *
 * attnqat_fwd_infer_mx_paged: q [B,Hq,Lq,d] bf16 holds the LAST Lq positions of every sequence; sequence b has
 * kv_lens[b] >= Lq keys (device int32 [B]) in the pages page_table[b*max_pages + 0 ..] (device int32 [B,max_pages],
 * max_pages >= ceil(max kv_len / 128)).  causal != 0: query i sees keys 0 .. kv_lens[b] - Lq + i (chunked prefill;
 * Lq = 1 is a decode step).  o [B,Hq,Lq,d] bf16, lse [B,Hq,Lq] fp32.  Page ids outside [0, num_pages) are clamped
 * (wrong result, no out-of-bounds access); a sequence with kv_lens[b] = 0 gets o = 0.
 */
size_t attnqat_kv_cache_page_bytes(int Hkv, int d);
int attnqat_kv_cache_write_mx(const void* k, const void* v, int Hkv, int L, int d, int dtype,
                              void* cache, int num_pages, const int* page_ids, void* stream);
int attnqat_fwd_infer_mx_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                               const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                               void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same serving setting in the paper's own format: an NVFP4 KV cache and Alg. 1 (attnqat_fwd_infer) over it.
 *
 * Cache: num_pages * attnqat_kv_cache_page_bytes_nvfp4(Hkv, d) bytes of caller-owned device memory.  A page holds 128
 * consecutive positions of one sequence for all Hkv heads; per head, in this order, K codes [128][d/2], K scale bytes
 * [128][d/16], V codes [128][d/2], V scale bytes [128][d/16]: the layout of attnqat_quantize (Eq. 1, blocks of 16 along
 * d) cut into pages, 4.5 bits per element.  Blocks do not span positions, so a sequence grows in place:
 *
 * attnqat_kv_cache_write quantizes k, v [1,Hkv,n,d] bf16, the n >= 1 positions pos0 .. pos0+n-1 of one sequence, into
 * the pages page_ids[pos / 128] (device int32; the sequence's page list from its first page on, ceil((pos0+n)/128)
 * entries) and clears the slots of the last page behind position pos0+n-1.  Slots before pos0 are left as they are.
 * A page id outside [0, num_pages) is not written (nothing outside the cache is touched).
 *
 * attnqat_fwd_infer_paged: arguments as attnqat_fwd_infer_mx_paged; kv_lens[b] must be >= 1, and >= Lq under the causal
 * mask (other values: that sequence's outputs are unspecified; no access outside the cache or the workspace).  Positions
 * of a page table entry outside [0, num_pages) read as zeros.  The result is attnqat_fwd_infer of every sequence on its
 * own (the last Lq rows of it), bit for bit when the pages hold what attnqat_quantize gives for K and V.
 * Workspace: attnqat_paged_workspace_bytes(B, Hq, Hkv, Lq, max_pages, d) (max_pages <= 8192); 0 for bad arguments.
 * cache must be 16-byte aligned.
 *
 * Two paths, chosen by the number of query rows per (sequence, kv head), (Hq / Hkv) * Lq:
 *   more than 16: the pages are unpacked into the fp16 K and V^T copies of attnqat_fwd_infer's kernel (the workspace
 *     holds them, laid out for max_pages * 128 positions per sequence), which then runs with per-sequence lengths.
 *   at most 16 (decode steps): one kernel reads the pages directly, once.  The keys of a sequence are cut into chunks
 *     that workgroups take from a queue (a small kernel in front lists the chunks that exist, from kv_lens and the page
 *     table as they are in memory when it runs), so that long sequences do not set the pace of the step.  P-tilde is quantized
 *     against the running maximum in key order (Alg. 1), which a chunk cannot know before the chunks in front of it have
 *     computed their scores: every chunk first computes its scores (the K half of its pages), publishes its row maxima
 *     in the workspace and waits for those of its predecessors, then does the rest (the V half).  Tickets are handed out
 *     in chunk order, so a predecessor is always running or finished when someone waits for it and the wait ends; it is
 *     bounded nevertheless (2^22 polls), and a wait that expired leaves a wrong result for that sequence.  The partial
 *     sums of the chunks of a sequence are added by a third kernel.  The result is not bit-identical to
 *     attnqat_fwd_infer (the sums are grouped differently) but holds the same parity bars against the oracle.
 * attnqat_debug_fwd_infer_paged is the same call with the poll limit as an argument (tests force the expiry path with
 * 0); it synchronizes the stream and sets *wait_expired (host) to 1 if any wait of the decode path ran out.
 */
size_t attnqat_kv_cache_page_bytes_nvfp4(int Hkv, int d);
int attnqat_kv_cache_write(const void* k, const void* v, int Hkv, int n, int d, int dtype, int pos0,
                           void* cache, int num_pages, const int* page_ids, void* stream);
size_t attnqat_paged_workspace_bytes(int B, int Hq, int Hkv, int Lq, int max_pages, int d);
int attnqat_fwd_infer_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                            const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                            void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);
int attnqat_debug_fwd_infer_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                                  const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                                  void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream,
                                  int spin_limit, int* wait_expired);

/*
 * Block-sparse attention (Sec. 5: the paper's datacenter inference kernel supports it): attnqat_fwd_infer_mx with a
 * block mask.  block_mask [B,Hq,nb,nb] bytes (device, read), nb = ceil(L/128): a zero byte removes the block of 128
 * queries x 128 keys, i.e. those keys count as masked for those queries and their key tiles are not visited (the
 * order of the remaining tiles, and with it the running maximum that P-tilde is quantized against, is unchanged).
 * The causal flag still applies inside the blocks that are kept.  A query without any key left gets o = 0 and
 * lse = -inf.  Workspace: ATTNQAT_WS_FWD_INFER_MX_SPARSE.
 */
int attnqat_fwd_infer_mx_sparse(const void* q, const void* k, const void* v,
                                int B, int Hq, int Hkv, int L, int d, int causal, int dtype, const uint8_t* block_mask,
                                void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Training forward (Alg. 2) and backward (Alg. 3) in the MX format, for training against
 * attnqat_fwd_infer_mx: the same quantizers (Q^F, K^F blocked along d; V^F, P-tilde^F and the
 * backward's recomputed P^F in blocks of 32 keys; power-of-two scales), O' from the un-quantized
 * P-tilde, D from O', dS from the fp32 P.  The score product S = Q^F K^F^T is computed from the codes and
 * scales by the FP4 matrix instruction in the forward and in both backward passes; the other products
 * (O and O' from V^F, dP, dS K, dS^T Q, P^F^T dO) run on the 16-bit matrix instructions with the dequantized
 * values (Eq. 4), which are the numbers the FP4 instruction multiplies (Eq. 3): O and lse agree with
 * attnqat_fwd_infer_mx up to fp32 summation order, except that dequantized values of P-tilde^F and V^F below
 * the fp16 range (2^-24; P-tilde^F far below the row maximum) are flushed here.  Arguments as attnqat_fwd / attnqat_bwd; workspace sizes ATTNQAT_WS_FWD_MX and
 * ATTNQAT_WS_BWD_MX.  attnqat_debug_fwd_p_mx is attnqat_debug_fwd_p for this forward.
 */
int attnqat_fwd_mx(const void* q, const void* k, const void* v,
                   int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                   void* o, float* lse, float* o_hp,
                   void* workspace, size_t workspace_bytes, void* stream);
int attnqat_bwd_mx(const void* q, const void* k, const void* v, const void* d_o,
                   const float* lse, const float* o_hp,
                   int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                   void* dq, void* dk, void* dv,
                   void* workspace, size_t workspace_bytes, void* stream);
int attnqat_debug_fwd_p_mx(const void* q, const void* k, const void* v,
                           int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                           void* o, float* lse, int row0, float* p_dump,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement hooks.  Their state is kept per stream: a setting made for one stream is seen only by entry points that are
 * later called with that same stream argument (NULL, the default stream, is a stream of its own here), so calls on
 * other streams and from other threads are not affected.  At most 16 streams can have a setting at a time
 * (ATTNQAT_EINVAL beyond that); switching a setting off frees nothing but is always accepted.
 *
 * attnqat_profile_enable / attnqat_profile_read: the kernels of Alg. 1-3 are enqueued back to back by one call, so a
 * caller cannot bracket a single kernel with its own events.  While enabled for `stream`, every entry point called on
 * it records a HIP event before its first kernel and after each kernel; the events are created on first use and kept
 * until the process ends (the one exception to "nothing is allocated").  attnqat_profile_read() must follow a
 * synchronisation of that stream; it returns the number of kernels of the most recent call on it and fills ms[i] with the
 * time between consecutive events and names[i] (may be NULL) with a static label.  Off by default.
 *
 * attnqat_debug_dkdv_tile_counts: the dK/dV pass of attnqat_bwd skips the work on P^F (quantizing it and
 * dV += P^F^T dO) for every 32-query x 32-key tile whose P^F is all zero, which is exact; how often that happens depends
 * on the data.  While `counts` (device, 2 x uint64, zeroed by the caller) is set for `stream`, every attnqat_bwd called
 * on it adds to counts[0] the number of tiles the pass visited and to counts[1] the number with a non-zero P^F.
 * NULL switches it off (the default).
 *
 * attnqat_debug_bwd_waves: the dQ and dK/dV passes run workgroups of 4 waves (128 query rows / 128 keys), and workgroups
 * of 8 waves (256) for the passes (NVFP4, with or without the options, and MX) of a problem large enough to keep two of
 * them per compute unit, under a causal mask only from 16384 positions on; both compute the same sums over the same tiles
 * in the same order.  waves = 4 or 8 forces one shape (8 only where that variant exists), 0 returns to
 * the automatic choice.  Process-wide, for tests that compare the two shapes at small sizes.  ATTNQAT_EINVAL for any
 * other value.
 */
int attnqat_profile_enable(void* stream, int on);
int attnqat_profile_read(void* stream, int max_entries, float* ms, const char** names);
int attnqat_debug_dkdv_tile_counts(void* stream, unsigned long long* counts);
int attnqat_debug_bwd_waves(int waves);

#ifdef __cplusplus
}
#endif
#endif /* ATTNQAT_H */
