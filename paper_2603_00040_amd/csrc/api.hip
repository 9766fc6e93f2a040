// extern "C" boundary: argument checks, workspace carving, kernel sequencing.
#include "../../include/attnqat.h"
#include "common.hpp"
#include "kernels.hpp"

#include <atomic>
#include <mutex>

using namespace aq;

// Scratch of attnqat_fwd_infer_static: the workspace of the inference forward as device memory that exists from the
// moment the library is loaded on a GPU until the process ends, so that the entry point never has to allocate.  Every
// GPU holds its own copy at its own address; in host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[ATTNQAT_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current GPU, looked up once per device (no allocation).  Null on failure.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;
void* static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Carver {
    unsigned char* base; size_t off;
    void* take(size_t bytes) { void* p = base ? base + off : nullptr; off += align_up(bytes); return p; }
};

// Measurement state, kept PER STREAM (a call only ever looks at the entry of the stream it enqueues on, so calls on
// different streams, from different threads, do not see each other's settings): optional per-kernel timing with HIP
// events recorded on the launch stream after every kernel, and the tile counters of the dK/dV pass.
struct StreamDbg {
    hipStream_t stream = nullptr;
    bool used = false;
    bool prof_on = false;
    bool created = false;
    int n = 0;
    hipEvent_t ev[16];
    const char* name[16];
    unsigned long long* dkdv_counts = nullptr;
};
constexpr int kMaxDbgStreams = 16;
StreamDbg g_dbg[kMaxDbgStreams];
std::mutex g_dbg_mutex;
std::atomic<int> g_dbg_active{0};          // entries with profiling on or a counter set: 0 = every call skips the table

// The entry of a stream; with create, a free entry is taken for it.  Caller holds g_dbg_mutex.
StreamDbg* dbg_entry(hipStream_t st, bool create)
{
    for (auto& e : g_dbg) if (e.used && e.stream == st) return &e;
    if (!create) return nullptr;
    for (auto& e : g_dbg) if (!e.used) { e.used = true; e.stream = st; return &e; }
    return nullptr;
}
void dbg_recount()
{
    int n = 0;
    for (auto& e : g_dbg) if (e.used && (e.prof_on || e.dkdv_counts)) ++n;
    g_dbg_active.store(n, std::memory_order_release);
}

void prof_begin(hipStream_t st)
{
    if (g_dbg_active.load(std::memory_order_acquire) == 0) return;
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry(st, false);
    if (!e || !e->prof_on) return;
    if (!e->created) {
        for (auto& v : e->ev) if (hipEventCreate(&v) != hipSuccess) { e->prof_on = false; dbg_recount(); return; }
        e->created = true;
    }
    e->n = 0;
    e->name[0] = "begin";
    (void)hipEventRecord(e->ev[e->n++], st);
}
void prof_mark(const char* name, hipStream_t st)
{
    if (g_dbg_active.load(std::memory_order_acquire) == 0) return;
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry(st, false);
    if (!e || !e->prof_on || e->n >= 16 || e->n == 0) return;
    e->name[e->n] = name;
    (void)hipEventRecord(e->ev[e->n++], st);
}
unsigned long long* dkdv_counts_of(hipStream_t st)
{
    if (g_dbg_active.load(std::memory_order_acquire) == 0) return nullptr;
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry(st, false);
    return e ? e->dkdv_counts : nullptr;
}

int check_dims(int B, int Hq, int Hkv, int L, int d, int dtype)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || L < 1) return ATTNQAT_EINVAL;
    if (dtype != ATTNQAT_BF16) return ATTNQAT_EDTYPE;
    if ((d != 64 && d != 128) || Hq % Hkv != 0) return ATTNQAT_ESHAPE;
    if (L > (1 << 20)) return ATTNQAT_ESHAPE;
    const long long nqt = (long long)round_up(L, kRowPad) / 128;
    if ((long long)B * Hq * nqt > 0x7FFFFFFFLL || (long long)B * Hq > 65535) return ATTNQAT_ESHAPE;
    return ATTNQAT_OK;
}

// Workspace of the forward: fp16 Q^F, K^F (row-major) and V^F^T.
struct FwdWs { void *qh, *kh, *vt, *tmp, *qsc; double* kpart; float* kmean; size_t bytes; };
FwdWs carve_fwd(void* ws, int B, int Hq, int Hkv, int L, int d, bool mx = false)
{
    const size_t Lp = round_up(L, kRowPad);
    Carver c{(unsigned char*)ws, 0};
    FwdWs w;
    w.qh = c.take((size_t)B * Hq * Lp * d * 2);
    w.kh = c.take((size_t)B * Hkv * Lp * d * 2);
    w.vt = c.take((size_t)B * Hkv * Lp * d * 2);
    w.tmp = mx ? c.take((size_t)B * Hq * L * d * 2) : nullptr;      // MX: the dequantized bf16 tensor before its layout copy
    // MX: qh and kh hold the operands of the FP4 instruction (smaller than the fp16 copies); the Q scale dwords come extra
    w.qsc = mx ? c.take(mx_qsc_bytes(B * Hq, L)) : nullptr;
    w.kpart = (double*)c.take(colmean_scratch_bytes(B * Hkv, d));  // K smoothing: partial sums and the token mean of K
    w.kmean = (float*)c.take((size_t)B * Hkv * d * 4);
    w.bytes = c.off;
    return w;
}

// Workspace of the backward: row-major copies (Q^F, K^F fp16; V^F and dO bf16: dO is not exactly
// representable in fp16), the per-row {L, D} pairs and the partial maxima that bound |dS|.
struct BwdWs { void *qb, *kb, *vb, *dob; float* rowstat; float* bounds; void* tmp; double* kpart; float* kmean; size_t bytes;
               void *qops, *qsc, *kops, *ksc, *krec; };
BwdWs carve_bwd(void* ws, int B, int Hq, int Hkv, int L, int d, bool mx = false)
{
    const size_t Lp = round_up(L, kRowPad);
    Carver c{(unsigned char*)ws, 0};
    BwdWs w;
    const size_t nq = (size_t)B * Hq * Lp * d * 2, nk = (size_t)B * Hkv * Lp * d * 2;
    w.qb = c.take(nq); w.kb = c.take(nk); w.vb = c.take(nk); w.dob = c.take(nq);
    w.rowstat = (float*)c.take((size_t)B * Hq * Lp * 8);
    w.bounds = (float*)c.take((size_t)3 * B * Hq * 64 * 4);
    w.tmp = mx ? c.take((size_t)B * Hq * L * d * 2) : nullptr;
    w.kpart = (double*)c.take(colmean_scratch_bytes(B * Hkv, d));
    w.kmean = (float*)c.take((size_t)B * Hkv * d * 4);
    // MX: the operand arrays of the FP4 instruction from which both passes recompute the scores
    w.qops = mx ? c.take(mx_qops_bytes(B * Hq, L, d)) : nullptr;
    w.qsc  = mx ? c.take(mx_qsc_bytes(B * Hq, L)) : nullptr;
    w.kops = mx ? c.take(mx_qops_bytes(B * Hkv, L, d)) : nullptr;
    w.ksc  = mx ? c.take(mx_qsc_bytes(B * Hkv, L)) : nullptr;
    w.krec = mx ? c.take(mx_ktrain_bytes(B * Hkv, L, d)) : nullptr;
    w.bytes = c.off;
    return w;
}

// Workspace of the MX forward: Q operand codes and scale dwords, and the 64-key kv records.
struct MxWs { unsigned char *qops, *qsc, *kv; size_t bytes; };
MxWs carve_mx(void* ws, int B, int Hq, int Hkv, int L, int d, bool fp8v = false)
{
    Carver c{(unsigned char*)ws, 0};
    MxWs w;
    w.qops = (unsigned char*)c.take(mx_qops_bytes(B * Hq, L, d));
    w.qsc = (unsigned char*)c.take(mx_qsc_bytes(B * Hq, L));
    w.kv = (unsigned char*)c.take(mx_kv_bytes(B * Hkv, L, d, fp8v));
    w.bytes = c.off;
    return w;
}

// phi of one input tensor and its layout copies (xr row-major, xt transposed; either may be null).
// NVFP4: one fused kernel.  MX: the MX fake-quantizer writes the dequantized bf16 tensor to tmp (blocks along d,
// or along the sequence for V), then the layout copy runs without quantizing.
int quant_copy(const void* x, int BH, int L, int d, bool mx, int mx_axis, bool out_f16, void* xr, void* xt, void* tmp, hipStream_t st,
               const float* sub = nullptr)
{
    if (!mx) return launch_prep(x, BH, L, d, true, out_f16, nullptr, nullptr, nullptr, xr, xt, st, sub);
    if (launch_mx_quant(x, BH, L, d, mx_axis, 0, false, nullptr, nullptr, tmp, st)) return -1;
    return launch_prep(tmp, BH, L, d, false, out_f16, nullptr, nullptr, nullptr, xr, xt, st);
}

int fwd_common(const void* q, const void* k, const void* v, int B, int Hq, int Hkv, int L, int d,
               int causal, int dtype, bool train, bool mx, void* o, float* lse, float* o_hp,
               int dump_row0, float* p_dump, void* workspace, size_t workspace_bytes, void* stream, int options = 0)
{
    if (!q || !k || !v || !o || !lse || (train && !o_hp)) return ATTNQAT_EINVAL;
    if ((options & ~(ATTNQAT_OPT_SMOOTH_K | ATTNQAT_OPT_TWO_LEVEL_P | ATTNQAT_OPT_BF16_PV)) || (options && mx)) return ATTNQAT_EINVAL;
    const bool bf16pv = (options & ATTNQAT_OPT_BF16_PV) != 0;
    if (bf16pv && (train || (options & ATTNQAT_OPT_TWO_LEVEL_P))) return ATTNQAT_EINVAL;     // an inference recipe; P has no blocks
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    FwdWs w = carve_fwd(workspace, B, Hq, Hkv, L, d, mx);
    if (!workspace || workspace_bytes < w.bytes) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    // Alg. 1 line "phi(Q), phi(K), phi(V)" / Alg. 2 line "Q^F, K^F, V^F"
    if (mx) {
        // Q and K as operands of the scaled FP4 instruction (the scores are computed from the codes), V^F^T as the fp16 copy
        if (launch_mx_quant(q, B * Hq, L, d, 0, 1, false, (unsigned char*)w.qh, (unsigned char*)w.qsc, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (launch_mx_quant(k, B * Hkv, L, d, 0, 3, false, (unsigned char*)w.kh, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (quant_copy(v, B * Hkv, L, d, true, 1, true, nullptr, w.vt, w.tmp, st)) return ATTNQAT_ELAUNCH;
        prof_mark("prep_qkv", st);
        if (launch_fwd(w.qh, w.kh, w.vt, B, Hq, Hkv, L, d, causal != 0, train, 1, o, lse, o_hp, dump_row0, p_dump, st, w.qsc))
            return ATTNQAT_ELAUNCH;
        prof_mark(train ? "fwd_train" : "fwd_infer", st);
        return ATTNQAT_OK;
    }
    if (quant_copy(q, B * Hq, L, d, mx, 0, true, w.qh, nullptr, w.tmp, st)) return ATTNQAT_ELAUNCH;
    const float* kmean = nullptr;
    if (options & ATTNQAT_OPT_SMOOTH_K) {          // K minus its token mean (Sec. 2.1), then phi
        if (launch_colmean(k, B * Hkv, L, d, w.kpart, w.kmean, st)) return ATTNQAT_ELAUNCH;
        kmean = w.kmean;
    }
    if (quant_copy(k, B * Hkv, L, d, mx, 0, true, w.kh, nullptr, w.tmp, st, kmean)) return ATTNQAT_ELAUNCH;
    if (bf16pv) {      // Sec. 2.5, NVFP4 Q K^T with BF16 P V: V only changes layout
        if (launch_prep(v, B * Hkv, L, d, false, false, nullptr, nullptr, nullptr, nullptr, w.vt, st)) return ATTNQAT_ELAUNCH;
    } else if (quant_copy(v, B * Hkv, L, d, mx, 1, true, nullptr, w.vt, w.tmp, st)) return ATTNQAT_ELAUNCH;
    prof_mark("prep_qkv", st);
    const int p_quant = mx ? 1 : bf16pv ? 3 : (options & ATTNQAT_OPT_TWO_LEVEL_P) ? 2 : 0;
    if (launch_fwd(w.qh, w.kh, w.vt, B, Hq, Hkv, L, d, causal != 0, train, p_quant, o, lse, o_hp, dump_row0, p_dump, st))
        return ATTNQAT_ELAUNCH;
    prof_mark(train ? "fwd_train" : "fwd_infer", st);
    return ATTNQAT_OK;
}

}  // namespace

extern "C" {

int attnqat_block_k(void) { return kBlockK; }

const char* attnqat_strerror(int code)
{
    switch (code) {
    case ATTNQAT_OK:         return "ok";
    case ATTNQAT_EINVAL:     return "invalid argument (null pointer or non-positive size)";
    case ATTNQAT_ESHAPE:     return "unsupported shape (d must be 64 or 128, Hq % Hkv == 0, L <= 2^20)";
    case ATTNQAT_EDTYPE:     return "unsupported dtype (only ATTNQAT_BF16)";
    case ATTNQAT_EWORKSPACE: return "workspace missing or too small (see attnqat_workspace_bytes)";
    case ATTNQAT_ELAUNCH:    return "kernel launch failed";
    case ATTNQAT_ESTATIC:    return "problem needs more scratch than ATTNQAT_STATIC_SCRATCH_BYTES (use the entry point that takes a workspace)";
    default:                 return "unknown error code";
    }
}

size_t attnqat_workspace_bytes(int which, int B, int Hq, int Hkv, int L, int d)
{
    if (check_dims(B, Hq, Hkv, L, d, ATTNQAT_BF16)) return 0;
    switch (which) {
    case ATTNQAT_WS_FWD:
    case ATTNQAT_WS_FWD_INFER: return carve_fwd(nullptr, B, Hq, Hkv, L, d).bytes;
    case ATTNQAT_WS_BWD:       return carve_bwd(nullptr, B, Hq, Hkv, L, d).bytes;
    case ATTNQAT_WS_FWD_INFER_MX: return carve_mx(nullptr, B, Hq, Hkv, L, d).bytes;
    case ATTNQAT_WS_FWD_INFER_MX_FP8PV: return carve_mx(nullptr, B, Hq, Hkv, L, d, true).bytes;
    case ATTNQAT_WS_FWD_INFER_MX_PAGED: {          // L = the number of query positions per sequence
        Carver c{nullptr, 0};
        c.take(mx_qops_bytes(B * Hq, L, d)); c.take(mx_qsc_bytes(B * Hq, L));
        return c.off;
    }
    case ATTNQAT_WS_FWD_INFER_MX_SPARSE: {
        const size_t nb = round_up(L, kRowPad) / 128, nrows = (size_t)B * Hq * nb;
        Carver c{nullptr, carve_mx(nullptr, B, Hq, Hkv, L, d, false).bytes};
        c.take(nrows * nb * 4); c.take(nrows * 4);
        return c.off;
    }
    case ATTNQAT_WS_FWD_MX:    return carve_fwd(nullptr, B, Hq, Hkv, L, d, true).bytes;
    case ATTNQAT_WS_BWD_MX:    return carve_bwd(nullptr, B, Hq, Hkv, L, d, true).bytes;
    default:                   return 0;
    }
}

int attnqat_quantize(const void* x, int B, int H, int L, int d, int dtype,
                     uint8_t* codes, uint8_t* scales, void* xf, void* stream)
{
    if (!x || (!codes && !scales && !xf)) return ATTNQAT_EINVAL;
    if (((uintptr_t)x & 15) || ((uintptr_t)codes & 7) || ((uintptr_t)scales & 3) || ((uintptr_t)xf & 15)) return ATTNQAT_EINVAL;
    int rc = check_dims(B, H, H, L, d, dtype);
    if (rc) return rc;
    prof_begin((hipStream_t)stream);
    if (launch_prep(x, B * H, L, d, true, false, codes, scales, xf, nullptr, nullptr, (hipStream_t)stream))
        return ATTNQAT_ELAUNCH;
    prof_mark("quantize", (hipStream_t)stream);
    return ATTNQAT_OK;
}

static int quantize_mx_common(const void* x, int B, int H, int L, int d, int dtype, int axis, bool fp8,
                              uint8_t* codes, uint8_t* scales, void* xf, void* stream)
{
    if (!x || (!codes && !scales && !xf) || (axis != 0 && axis != 1) || (fp8 && axis != 1)) return ATTNQAT_EINVAL;
    int rc = check_dims(B, H, H, L, d, dtype);
    if (rc) return rc;
    prof_begin((hipStream_t)stream);
    if (launch_mx_quant(x, B * H, L, d, axis, 0, fp8, codes, scales, xf, (hipStream_t)stream)) return ATTNQAT_ELAUNCH;
    prof_mark("quantize_mx", (hipStream_t)stream);
    return ATTNQAT_OK;
}

int attnqat_quantize_mx(const void* x, int B, int H, int L, int d, int dtype, int axis,
                        uint8_t* codes, uint8_t* scales, void* xf, void* stream)
{
    return quantize_mx_common(x, B, H, L, d, dtype, axis, false, codes, scales, xf, stream);
}

int attnqat_quantize_mxfp8(const void* x, int B, int H, int L, int d, int dtype, int axis,
                           uint8_t* codes, uint8_t* scales, void* xf, void* stream)
{
    return quantize_mx_common(x, B, H, L, d, dtype, axis, true, codes, scales, xf, stream);
}

static int fwd_infer_mx_common(const void* q, const void* k, const void* v,
                               int B, int Hq, int Hkv, int L, int d, int causal, int dtype, bool fp8pv,
                               void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !o || !lse) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    MxWs w = carve_mx(workspace, B, Hq, Hkv, L, d, fp8pv);
    if (!workspace || workspace_bytes < w.bytes) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    // Alg. 1 first line, in the MX format: phi(Q), phi(K) along d, phi(V) along the keys (E4M3 elements in the mixed recipe)
    if (launch_mx_quant(q, B * Hq, L, d, 0, 1, false, w.qops, w.qsc, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_mx_quant(k, B * Hkv, L, d, 0, 2, fp8pv, w.kv, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_mx_quant(v, B * Hkv, L, d, 1, 2, fp8pv, w.kv, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
    prof_mark("prep_qkv_mx", st);
    if (launch_fwd_mx(w.qops, w.qsc, w.kv, B, Hq, Hkv, L, d, causal != 0, fp8pv, o, lse, st)) return ATTNQAT_ELAUNCH;
    prof_mark(fp8pv ? "fwd_infer_mx_fp8pv" : "fwd_infer_mx", st);
    return ATTNQAT_OK;
}

int attnqat_fwd_infer_mx(const void* q, const void* k, const void* v,
                         int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                         void* o, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_infer_mx_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, o, lse, workspace, workspace_bytes, stream);
}

int attnqat_fwd_infer_mx_fp8pv(const void* q, const void* k, const void* v,
                               int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                               void* o, float* lse,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_infer_mx_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, true, o, lse, workspace, workspace_bytes, stream);
}

int attnqat_fwd_infer_mx_sparse(const void* q, const void* k, const void* v,
                                int B, int Hq, int Hkv, int L, int d, int causal, int dtype, const uint8_t* block_mask,
                                void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !o || !lse || !block_mask) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    const size_t nb = round_up(L, kRowPad) / 128, nrows = (size_t)B * Hq * nb;
    MxWs w = carve_mx(workspace, B, Hq, Hkv, L, d, false);
    Carver c{(unsigned char*)workspace, w.bytes};
    int* list = (int*)c.take(nrows * nb * 4);
    int* cnt = (int*)c.take(nrows * 4);
    if (!workspace || workspace_bytes < c.off) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (launch_mx_quant(q, B * Hq, L, d, 0, 1, false, w.qops, w.qsc, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_mx_quant(k, B * Hkv, L, d, 0, 2, false, w.kv, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_mx_quant(v, B * Hkv, L, d, 1, 2, false, w.kv, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
    prof_mark("prep_qkv_mx", st);
    if (launch_fwd_mx_sparse(w.qops, w.qsc, w.kv, B, Hq, Hkv, L, d, causal != 0, block_mask, list, cnt, o, lse, st)) return ATTNQAT_ELAUNCH;
    prof_mark("fwd_infer_mx_sparse", st);
    return ATTNQAT_OK;
}

size_t attnqat_kv_cache_page_bytes(int Hkv, int d)
{
    if (Hkv < 1 || (d != 64 && d != 128)) return 0;
    return (size_t)Hkv * mx_page_bytes(d);
}

int attnqat_kv_cache_write_mx(const void* k, const void* v, int Hkv, int L, int d, int dtype,
                              void* cache, int num_pages, const int* page_ids, void* stream)
{
    if (!k || !v || !cache || !page_ids || num_pages < 1) return ATTNQAT_EINVAL;
    int rc = check_dims(1, Hkv, Hkv, L, d, dtype);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (launch_mx_quant(k, Hkv, L, d, 0, 2, false, (unsigned char*)cache, nullptr, nullptr, st, page_ids, num_pages)) return ATTNQAT_ELAUNCH;
    if (launch_mx_quant(v, Hkv, L, d, 1, 2, false, (unsigned char*)cache, nullptr, nullptr, st, page_ids, num_pages)) return ATTNQAT_ELAUNCH;
    prof_mark("kv_cache_write_mx", st);
    return ATTNQAT_OK;
}

int attnqat_fwd_infer_mx_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                               const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                               void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !cache || !page_table || !kv_lens || !o || !lse || num_pages < 1 || max_pages < 1) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, Lq, d, dtype);
    if (rc) return rc;
    // Grouped-query heads with few positions: q [B,Hq,Lq,d] is [B*Hkv, G*Lq, d] in memory, so the G query heads of a kv
    // group are treated as one head with G*Lq rows: one tile and one pass over the pages instead of G.
    const int G = Hq / Hkv;
    const bool pack = G > 1 && G * Lq <= 128;
    const int Hq_k = pack ? Hkv : Hq, Lq_k = pack ? G * Lq : Lq;
    Carver c{(unsigned char*)workspace, 0};
    unsigned char* qops = (unsigned char*)c.take(mx_qops_bytes(B * Hq, Lq, d));      // sized for the unpacked case (the larger)
    unsigned char* qsc = (unsigned char*)c.take(mx_qsc_bytes(B * Hq, Lq));
    if (!workspace || workspace_bytes < c.off) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (launch_mx_quant(q, B * Hq_k, Lq_k, d, 0, 1, false, qops, qsc, nullptr, st)) return ATTNQAT_ELAUNCH;
    prof_mark("prep_q_mx", st);
    if (launch_fwd_mx_paged(qops, qsc, cache, B, Hq_k, Hkv, Lq_k, d, causal != 0, page_table, kv_lens, max_pages, num_pages, Lq, o, lse, st))
        return ATTNQAT_ELAUNCH;
    prof_mark("fwd_infer_mx_paged", st);
    return ATTNQAT_OK;
}

size_t attnqat_kv_cache_page_bytes_nvfp4(int Hkv, int d)
{
    if (Hkv < 1 || (d != 64 && d != 128)) return 0;
    return nvfp4_page_bytes(Hkv, d);
}

int attnqat_kv_cache_write(const void* k, const void* v, int Hkv, int n, int d, int dtype, int pos0,
                           void* cache, int num_pages, const int* page_ids, void* stream)
{
    if (!k || !v || !cache || !page_ids || num_pages < 1 || pos0 < 0) return ATTNQAT_EINVAL;
    int rc = check_dims(1, Hkv, Hkv, n, d, dtype);
    if (rc) return rc;
    if ((long long)pos0 + n > (1 << 20)) return ATTNQAT_ESHAPE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (launch_kv_page_write(k, v, Hkv, n, d, pos0, cache, num_pages, page_ids, st)) return ATTNQAT_ELAUNCH;
    prof_mark("kv_cache_write", st);
    return ATTNQAT_OK;
}

namespace {
// Few rows per (sequence, kv head): the decode kernel reads the pages itself (dec != null); otherwise the pages are unpacked
// into the K / V^T copies of the general forward.
struct PagedWs { void *qh, *kh, *vt, *dec; size_t bytes; int Lkp; };
PagedWs carve_paged(void* ws, int B, int Hq, int Hkv, int Lq, int max_pages, int d)
{
    Carver c{(unsigned char*)ws, 0};
    PagedWs w{};
    const int R = (Hq / Hkv) * Lq;
    if (R <= decode_max_rows()) {
        w.qh = c.take((size_t)B * Hkv * kRowPad * d * 2);
        w.dec = c.take(decode_ws_bytes(B, Hkv, R, max_pages, d));
    } else {
        w.Lkp = (int)round_up(max_pages * 128, kRowPad);
        w.qh = c.take((size_t)B * Hq * round_up(Lq, kRowPad) * d * 2);
        w.kh = c.take((size_t)B * Hkv * w.Lkp * d * 2);
        w.vt = c.take((size_t)B * Hkv * w.Lkp * d * 2);
    }
    w.bytes = c.off;
    return w;
}

constexpr int kDecodeSpinLimit = 1 << 22;       // polls (each at least a microsecond apart) before a chunk gives up waiting

int paged_common(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                 const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                 void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream, int spin_limit, void** dec_ws)
{
    if (!q || !cache || !page_table || !kv_lens || !o || !lse || num_pages < 1 || max_pages < 1) return ATTNQAT_EINVAL;
    if ((uintptr_t)cache & 15) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, Lq, d, dtype);
    if (rc) return rc;
    if (max_pages > (1 << 13) || (long long)B * Hkv > 65535) return ATTNQAT_ESHAPE;          // 2^20 keys per sequence
    PagedWs w = carve_paged(workspace, B, Hq, Hkv, Lq, max_pages, d);
    if (!workspace || workspace_bytes < w.bytes) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (w.dec) {
        // q [B,Hq,Lq,d] is [B*Hkv, G*Lq, d] in memory: the rows of a kv group form one tile
        if (launch_prep(q, B * Hkv, (Hq / Hkv) * Lq, d, true, true, nullptr, nullptr, nullptr, w.qh, nullptr, st)) return ATTNQAT_ELAUNCH;
        prof_mark("prep_q", st);
        if (launch_decode(w.qh, cache, num_pages, page_table, max_pages, kv_lens, B, Hq, Hkv, Lq, d, causal != 0, w.dec, spin_limit, o, lse, st))
            return ATTNQAT_ELAUNCH;
        prof_mark("decode_paged", st);
        if (dec_ws) *dec_ws = w.dec;
        return ATTNQAT_OK;
    }
    if (dec_ws) *dec_ws = nullptr;
    // phi(Q); K^F and V^F are in the cache already and only change layout
    if (launch_prep(q, B * Hq, Lq, d, true, true, nullptr, nullptr, nullptr, w.qh, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_unpack_pages(cache, page_table, kv_lens, B, Hkv, max_pages, num_pages, d, 0, w.kh, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_unpack_pages(cache, page_table, kv_lens, B, Hkv, max_pages, num_pages, d, 1, nullptr, w.vt, st)) return ATTNQAT_ELAUNCH;
    prof_mark("prep_q_unpack_pages", st);
    if (launch_fwd_varlen(w.qh, w.kh, w.vt, B, Hq, Hkv, Lq, w.Lkp, d, causal != 0, kv_lens, o, lse, st)) return ATTNQAT_ELAUNCH;
    prof_mark("fwd_infer_paged", st);
    return ATTNQAT_OK;
}
}  // namespace

size_t attnqat_paged_workspace_bytes(int B, int Hq, int Hkv, int Lq, int max_pages, int d)
{
    if (check_dims(B, Hq, Hkv, Lq, d, ATTNQAT_BF16) || max_pages < 1 || max_pages > (1 << 13)) return 0;
    return carve_paged(nullptr, B, Hq, Hkv, Lq, max_pages, d).bytes;
}

int attnqat_fwd_infer_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                            const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                            void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    return paged_common(q, B, Hq, Hkv, Lq, d, causal, dtype, cache, num_pages, page_table, max_pages, kv_lens, o, lse,
                        workspace, workspace_bytes, stream, kDecodeSpinLimit, nullptr);
}

int attnqat_debug_fwd_infer_paged(const void* q, int B, int Hq, int Hkv, int Lq, int d, int causal, int dtype,
                                  const void* cache, int num_pages, const int* page_table, int max_pages, const int* kv_lens,
                                  void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream,
                                  int spin_limit, int* wait_expired)
{
    if (spin_limit < 0 || !wait_expired) return ATTNQAT_EINVAL;
    void* dec = nullptr;
    int rc = paged_common(q, B, Hq, Hkv, Lq, d, causal, dtype, cache, num_pages, page_table, max_pages, kv_lens, o, lse,
                          workspace, workspace_bytes, stream, spin_limit, &dec);
    if (rc) return rc;
    *wait_expired = 0;
    if (dec) {
        if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ATTNQAT_ELAUNCH;
        if (hipMemcpy(wait_expired, (const unsigned char*)dec + 4, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return ATTNQAT_ELAUNCH;
    }
    return ATTNQAT_OK;
}

int attnqat_debug_dkdv_tile_counts(void* stream, unsigned long long* counts)
{
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry((hipStream_t)stream, counts != nullptr);
    if (!e) return counts ? ATTNQAT_EINVAL : ATTNQAT_OK;       // no free entry / nothing to switch off
    e->dkdv_counts = counts;
    dbg_recount();
    return ATTNQAT_OK;
}

int attnqat_debug_bwd_waves(int waves)
{
    if (waves != 0 && waves != 4 && waves != 8) return ATTNQAT_EINVAL;
    aq::set_bwd_waves(waves);
    return ATTNQAT_OK;
}

int attnqat_profile_enable(void* stream, int on)
{
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry((hipStream_t)stream, on != 0);
    if (!e) return on ? ATTNQAT_EINVAL : ATTNQAT_OK;
    e->prof_on = on != 0;
    e->n = 0;
    dbg_recount();
    return ATTNQAT_OK;
}

int attnqat_profile_read(void* stream, int max_entries, float* ms, const char** names)
{
    if (!ms || max_entries < 1) return ATTNQAT_EINVAL;
    std::lock_guard<std::mutex> lock(g_dbg_mutex);
    StreamDbg* e = dbg_entry((hipStream_t)stream, false);
    if (!e) return 0;
    int n = 0;
    for (int i = 1; i < e->n && n < max_entries; ++i, ++n) {
        if (hipEventElapsedTime(&ms[n], e->ev[i - 1], e->ev[i]) != hipSuccess) return ATTNQAT_ELAUNCH;
        if (names) names[n] = e->name[i];
    }
    return n;
}

int attnqat_fwd(const void* q, const void* k, const void* v,
                int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                void* o, float* lse, float* o_hp,
                void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, true, false, o, lse, o_hp, 0, nullptr,
                      workspace, workspace_bytes, stream);
}

int attnqat_fwd_infer(const void* q, const void* k, const void* v,
                      int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                      void* o, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, false, o, lse, nullptr, 0, nullptr,
                      workspace, workspace_bytes, stream);
}

int attnqat_fwd_infer_static(const void* q, const void* k, const void* v,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* stream)
{
    if (!q || !k || !v || !o || !lse) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    const size_t need = carve_fwd(nullptr, B, Hq, Hkv, L, d).bytes;
    if (need > (size_t)ATTNQAT_STATIC_SCRATCH_BYTES) return ATTNQAT_ESTATIC;
    void* ws = static_scratch_of_current_device();       // the device address, never the array's name
    if (!ws) return ATTNQAT_ELAUNCH;
    // Nothing has to start at zero: the quantization pass writes every byte of the copies that the forward reads
    // (padding rows included) before the forward runs, whatever an earlier call left behind.
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, false, o, lse, nullptr, 0, nullptr,
                      ws, need, stream);
}

int attnqat_fwd_infer_packed(const uint8_t* q_codes, const uint8_t* q_scales, const uint8_t* k_codes, const uint8_t* k_scales,
                             const uint8_t* v_codes, const uint8_t* v_scales,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q_codes || !q_scales || !k_codes || !k_scales || !v_codes || !v_scales || !o || !lse) return ATTNQAT_EINVAL;
    if (((uintptr_t)q_codes | (uintptr_t)k_codes | (uintptr_t)v_codes) & 7) return ATTNQAT_EINVAL;
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    FwdWs w = carve_fwd(workspace, B, Hq, Hkv, L, d);
    if (!workspace || workspace_bytes < w.bytes) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    // Alg. 1 takes the quantized tensors: only the layout copies remain to be made
    if (launch_unpack(q_codes, q_scales, B * Hq, L, d, true, w.qh, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_unpack(k_codes, k_scales, B * Hkv, L, d, true, w.kh, nullptr, st)) return ATTNQAT_ELAUNCH;
    if (launch_unpack(v_codes, v_scales, B * Hkv, L, d, true, nullptr, w.vt, st)) return ATTNQAT_ELAUNCH;
    prof_mark("unpack_qkv", st);
    if (launch_fwd(w.qh, w.kh, w.vt, B, Hq, Hkv, L, d, causal != 0, false, 0, o, lse, nullptr, 0, nullptr, st)) return ATTNQAT_ELAUNCH;
    prof_mark("fwd_infer", st);
    return ATTNQAT_OK;
}

int attnqat_debug_fwd_p(const void* q, const void* k, const void* v,
                        int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                        void* o, float* lse, int row0, float* p_dump,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!p_dump || row0 < 0 || row0 % 128 != 0) return ATTNQAT_EINVAL;
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, false, o, lse, nullptr, row0, p_dump,
                      workspace, workspace_bytes, stream);
}

int attnqat_fwd_opt(const void* q, const void* k, const void* v,
                    int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                    void* o, float* lse, float* o_hp,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, o_hp != nullptr, false, o, lse, o_hp, 0, nullptr,
                      workspace, workspace_bytes, stream, options);
}

int attnqat_fwd_infer_bf16pv(const void* q, const void* k, const void* v,
                             int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                             void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, false, o, lse, nullptr, 0, nullptr,
                      workspace, workspace_bytes, stream, ATTNQAT_OPT_BF16_PV);
}

int attnqat_debug_fwd_p_opt(const void* q, const void* k, const void* v,
                            int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                            void* o, float* lse, int row0, float* p_dump,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!p_dump || row0 < 0 || row0 % 128 != 0) return ATTNQAT_EINVAL;
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, false, o, lse, nullptr, row0, p_dump,
                      workspace, workspace_bytes, stream, options);
}

int attnqat_fwd_mx(const void* q, const void* k, const void* v,
                   int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                   void* o, float* lse, float* o_hp,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, true, true, o, lse, o_hp, 0, nullptr,
                      workspace, workspace_bytes, stream);
}

int attnqat_debug_fwd_p_mx(const void* q, const void* k, const void* v,
                           int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                           void* o, float* lse, int row0, float* p_dump,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (!p_dump || row0 < 0 || row0 % 128 != 0) return ATTNQAT_EINVAL;
    return fwd_common(q, k, v, B, Hq, Hkv, L, d, causal, dtype, false, true, o, lse, nullptr, row0, p_dump,
                      workspace, workspace_bytes, stream);
}

// The six arrays of an already quantized Q, K, V (attnqat_quantize's layout); null = quantize q, k, v here.
struct PackedQKV { const uint8_t *qc, *qs, *kc, *ks, *vc, *vs; };

static int bwd_common(const void* q, const void* k, const void* v, const void* d_o,
                      const float* lse, const void* o_acc, bool o_is_bf16, int p_quant /* 0 none, 1 NVFP4, 2 MX; 3 (two-level) is set from the options */,
                      int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                      void* dq, void* dk, void* dv,
                      void* workspace, size_t workspace_bytes, void* stream, int options = 0, const PackedQKV* packed = nullptr,
                      float* p_dump = nullptr, int dump_row0 = 0)
{
    if (p_dump && (p_quant != 1 || (options & ATTNQAT_OPT_TWO_LEVEL_P))) return ATTNQAT_EINVAL;
    if (packed) {
        if (!packed->qc || !packed->qs || !packed->kc || !packed->ks || !packed->vc || !packed->vs) return ATTNQAT_EINVAL;
        if (((uintptr_t)packed->qc | (uintptr_t)packed->kc | (uintptr_t)packed->vc) & 7) return ATTNQAT_EINVAL;
        if (options || p_quant != 1) return ATTNQAT_EINVAL;
        q = packed->qc; k = packed->kc; v = packed->vc;            // for the null checks below
    }
    if (!q || !k || !v || !d_o || !lse || !o_acc || !dq || !dk || !dv) return ATTNQAT_EINVAL;
    if ((options & ~(ATTNQAT_OPT_SMOOTH_K | ATTNQAT_OPT_TWO_LEVEL_P)) || (options && p_quant != 1)) return ATTNQAT_EINVAL;
    if (options & ATTNQAT_OPT_TWO_LEVEL_P) p_quant = 3;
    int rc = check_dims(B, Hq, Hkv, L, d, dtype);
    if (rc) return rc;
    const bool mx = p_quant == 2;
    BwdWs w = carve_bwd(workspace, B, Hq, Hkv, L, d, mx);
    if (!workspace || workspace_bytes < w.bytes) return ATTNQAT_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    prof_begin(st);
    if (packed) {
        // the saved quantized tensors of the forward (appendix "Detailed Training Setup": the extra buffers for the
        // fake-quantized Q, K, V): only the layout copies remain to be made
        if (launch_unpack(packed->qc, packed->qs, B * Hq, L, d, true, w.qb, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (launch_unpack(packed->kc, packed->ks, B * Hkv, L, d, true, w.kb, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (launch_unpack(packed->vc, packed->vs, B * Hkv, L, d, false, w.vb, nullptr, st)) return ATTNQAT_ELAUNCH;
    } else {
    // Q^F, K^F, V^F again (bit-identical to the forward's) and a zero-padded copy of dO
    if (quant_copy(q, B * Hq, L, d, mx, 0, true, w.qb, nullptr, w.tmp, st)) return ATTNQAT_ELAUNCH;
    const float* kmean = nullptr;
    if (options & ATTNQAT_OPT_SMOOTH_K) {          // the same centred K as the forward (deterministic mean)
        if (launch_colmean(k, B * Hkv, L, d, w.kpart, w.kmean, st)) return ATTNQAT_ELAUNCH;
        kmean = w.kmean;
    }
    if (quant_copy(k, B * Hkv, L, d, mx, 0, true, w.kb, nullptr, w.tmp, st, kmean)) return ATTNQAT_ELAUNCH;
    if (quant_copy(v, B * Hkv, L, d, mx, 1, false, w.vb, nullptr, w.tmp, st)) return ATTNQAT_ELAUNCH;
    }
    if (launch_prep(d_o, B * Hq, L, d, false, false, nullptr, nullptr, nullptr, w.dob, nullptr, st)) return ATTNQAT_ELAUNCH;
    MxScoreOps mxo{w.qops, w.qsc, w.kops, w.ksc, w.krec};
    if (mx) {
        if (launch_mx_quant(q, B * Hq, L, d, 0, 1, false, (unsigned char*)w.qops, (unsigned char*)w.qsc, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (launch_mx_quant(k, B * Hkv, L, d, 0, 1, false, (unsigned char*)w.kops, (unsigned char*)w.ksc, nullptr, st)) return ATTNQAT_ELAUNCH;
        if (launch_mx_quant(k, B * Hkv, L, d, 0, 3, false, (unsigned char*)w.krec, nullptr, nullptr, st)) return ATTNQAT_ELAUNCH;
    }
    prof_mark("prep_qkvdo", st);
    if (launch_delta(d_o, o_acc, o_is_bf16, lse, B * Hq, L, d, w.rowstat, st)) return ATTNQAT_ELAUNCH;
    prof_mark("delta", st);
    if (launch_bounds(w.vb, w.dob, w.rowstat, B * Hkv, B * Hq, L, d, w.bounds, st)) return ATTNQAT_ELAUNCH;
    prof_mark("bounds", st);
    if (launch_bwd_dq(w.qb, w.kb, w.vb, w.dob, w.rowstat, w.bounds, B, Hq, Hkv, L, d, causal != 0, dq, st, mx ? &mxo : nullptr))
        return ATTNQAT_ELAUNCH;
    prof_mark("bwd_dq", st);
    if (launch_bwd_dkdv(w.qb, w.kb, w.vb, w.dob, w.rowstat, w.bounds, B, Hq, Hkv, L, d, causal != 0, dk, dv,
                        dkdv_counts_of(st), p_quant, st, p_dump, dump_row0, mx ? &mxo : nullptr))
        return ATTNQAT_ELAUNCH;
    prof_mark("bwd_dkdv", st);
    return ATTNQAT_OK;
}

int attnqat_bwd(const void* q, const void* k, const void* v, const void* d_o,
                const float* lse, const float* o_hp,
                int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                void* dq, void* dk, void* dv,
                void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_common(q, k, v, d_o, lse, o_hp, false, 1, B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv,
                      workspace, workspace_bytes, stream);
}

int attnqat_bwd_packed(const uint8_t* q_codes, const uint8_t* q_scales, const uint8_t* k_codes, const uint8_t* k_scales,
                       const uint8_t* v_codes, const uint8_t* v_scales, const void* d_o,
                       const float* lse, const float* o_hp,
                       int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                       void* dq, void* dk, void* dv,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    const PackedQKV pk{q_codes, q_scales, k_codes, k_scales, v_codes, v_scales};
    return bwd_common(nullptr, nullptr, nullptr, d_o, lse, o_hp, false, 1, B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv,
                      workspace, workspace_bytes, stream, 0, &pk);
}

int attnqat_bwd_opt(const void* q, const void* k, const void* v, const void* d_o,
                    const float* lse, const float* o_hp,
                    int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int options,
                    void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_common(q, k, v, d_o, lse, o_hp, false, 1, B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv,
                      workspace, workspace_bytes, stream, options);
}

int attnqat_debug_bwd_p(const void* q, const void* k, const void* v, const void* d_o,
                        const float* lse, const float* o_hp,
                        int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                        void* dq, void* dk, void* dv, int row0, float* p_dump,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!p_dump || row0 < 0 || row0 % 128 != 0) return ATTNQAT_EINVAL;
    return bwd_common(q, k, v, d_o, lse, o_hp, false, 1, B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv,
                      workspace, workspace_bytes, stream, 0, nullptr, p_dump, row0);
}

int attnqat_bwd_mx(const void* q, const void* k, const void* v, const void* d_o,
                   const float* lse, const float* o_hp,
                   int B, int Hq, int Hkv, int L, int d, int causal, int dtype,
                   void* dq, void* dk, void* dv,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_common(q, k, v, d_o, lse, o_hp, false, 2, B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv,
                      workspace, workspace_bytes, stream);
}

int attnqat_bwd_ablation(const void* q, const void* k, const void* v, const void* d_o,
                         const float* lse, const float* o_hp, const void* o,
                         int B, int Hq, int Hkv, int L, int d, int causal, int dtype, int ablation,
                         void* dq, void* dk, void* dv,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    if (ablation & ~(ATTNQAT_ABL_D_FROM_O | ATTNQAT_ABL_P_UNQUANTIZED)) return ATTNQAT_EINVAL;
    const bool low = (ablation & ATTNQAT_ABL_D_FROM_O) != 0;
    return bwd_common(q, k, v, d_o, lse, low ? o : (const void*)o_hp, low, (ablation & ATTNQAT_ABL_P_UNQUANTIZED) ? 0 : 1,
                      B, Hq, Hkv, L, d, causal, dtype, dq, dk, dv, workspace, workspace_bytes, stream);
}

}  // extern "C"
