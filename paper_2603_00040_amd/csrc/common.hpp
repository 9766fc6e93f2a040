// Shared device helpers for the gfx950 Attn-QAT kernels: vector types, the
// NVFP4 rounding primitives (Sec. 2.1, Eq. 1-2) and the MFMA operand layouts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aq {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

constexpr int kBlockK = 64;      // semantic key tile B_k of Alg. 1/2
constexpr int kRowPad = 128;     // sequence lengths are padded to this in workspace copies

__host__ __device__ inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// ---- bf16 <-> fp32 (bit exact) -------------------------------------------
__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ inline uint32_t pack_bf16x2_rne(float lo, float hi) {
    return (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
}
// The same rounding by the conversion instruction of gfx950 (one instruction per pair; finite inputs give the same bits).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16x2_cvt(float lo, float hi) {
    const bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}
__device__ inline uint32_t pack_f16x2(float lo, float hi) {
    half2v h; h[0] = (half_t)lo; h[1] = (half_t)hi;      // RNE conversions
    return __builtin_bit_cast(uint32_t, h);
}

// ---- NVFP4 rounding --------------------------------------------------------
// Round v >= 0 to the E4M3 grid (RNE; subnormal spacing 2^-9 below 2^-6) by adding
// and subtracting 1.5 * 2^(e+20): an fp32 add rounds to nearest-even at exactly the
// E4M3 spacing of v's binade.  The caller clamps to 448.
__device__ inline float rne_e4m3_grid(float v) {
    uint32_t e = __float_as_uint(v) & 0x7F800000u;
    e = e > 0x3C800000u ? e : 0x3C800000u;                 // binades below 2^-6 share 2^-6's spacing
    float c = __uint_as_float(e + 0x0A400000u);            // 1.5 * 2^(e+20)
    return (v + c) - c;
}
// Round 0 <= r <= 6 to the E2M1 grid {0,.5,1,1.5,2,3,4,6} (RNE), same trick with
// 1.5 * 2^(e+22); binades below 1 share the spacing 0.5.
__device__ inline float rne_e2m1_grid(float r) {
    uint32_t e = __float_as_uint(r) & 0x7F800000u;
    e = e > 0x3F800000u ? e : 0x3F800000u;
    float c = __uint_as_float(e + 0x0B400000u);            // 1.5 * 2^(e+22)
    return (r + c) - c;
}
// E4M3 byte of a value already on the E4M3 grid (0 <= s <= 448).
__device__ inline uint32_t e4m3_byte_of(float s) {
    uint32_t u = __float_as_uint(s);
    if (s < 0.015625f) return (uint32_t)(s * 512.0f);      // subnormal: m * 2^-9
    return (((u >> 23) - 120u) << 3) | ((u >> 20) & 7u);
}
// E2M1 magnitude index (0..7) of a value already on the E2M1 grid.
__device__ inline uint32_t e2m1_index_of(float q) {
    return q < 1.0f ? (uint32_t)(q * 2.0f) : (__float_as_uint(q) >> 22) - 252u;
}

// Block scale of Eq. 1, exact: RNE_E4M3(amax/6) saturating at 448.  amax/6 is an IEEE
// (correctly rounded) division; for bf16 amax no quotient lies within 2^-13 (relative)
// of an E4M3 rounding boundary without being on it, so rounding the fp32 quotient
// equals rounding the real one.
__device__ inline float block_scale_exact(float amax) {
    float v = amax / 6.0f;
    v = v < 448.0f ? v : 448.0f;
    return rne_e4m3_grid(v);
}

// ---- MX format (E2M1 blocks of 32, power-of-two E8M0 scale) -------------------
// E8M0 byte of the smallest power of two s >= 2^-126 with 6 s >= amax (amax >= 0, finite).
// With amax = m 2^x, 1 <= m < 2:  6 * 2^(x-2) = 1.5 * 2^x covers m <= 1.5, else one more.
__device__ inline uint32_t e8m0_of_amax(float amax) {
    const uint32_t b = (__float_as_uint(amax) + 0x003FFFFFu) >> 23;      // biased exponent, +1 if mantissa > 1.5
    return b > 3u ? b - 2u : 1u;
}
// The same for E4M3 elements: the smallest power of two s >= 2^-126 with 448 s >= amax (448 = 1.75 * 2^8).
__device__ inline uint32_t e8m0_of_amax_fp8(float amax) {
    const uint32_t b = (__float_as_uint(amax) + 0x001FFFFFu) >> 23;      // biased exponent, +1 if mantissa > 1.75
    return b > 9u ? b - 8u : 1u;
}
__device__ inline float e8m0_as_f32(uint32_t byte) { return __uint_as_float(byte << 23); }            // 1 <= byte <= 254
__device__ inline float e8m0_inverse_as_f32(uint32_t byte) { return __uint_as_float((254u - byte) << 23); }   // 1 <= byte <= 253

// Bytes of one 64-key K record of the MX training forward (operands of the scaled FP4 instruction and their scale dwords).
__host__ __device__ constexpr int mx_ktrain_rec_bytes(int D) { return 2 * (D / 64) * 1024 + 1024; }

// The result of v_mfma_scale_f32_32x32x64_f8f6f4 must not be read by a vector instruction before the wait states of the matrix
// pipeline have passed; the compiler counts them inside a basic block, but when the product is the last instruction of a
// block it inserts nothing at the start of the next one (seen: the first score register read too early, NaN).  These
// no-ops, tied to the accumulators by a data dependence, stand behind the last score product of a tile in every kernel
// that uses the instruction on the 16-bit path.
__device__ inline void mfma_scale_settle(floatx16& a) { asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a)); }
__device__ inline void mfma_scale_settle(floatx16& a, floatx16& b) { asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a), "+v"(b)); }

// max(a, b) written as median(a, b, +inf): fmaxf() on values the compiler cannot prove quiet (MFMA
// results) costs a canonicalizing v_max per operand, the median has no such requirement and the
// compiler folds chains of it into v_max3.  No NaN reaches these reductions.
__device__ inline float max_nc(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, __builtin_inff()); }
// A lone two-input maximum still gets its operands canonicalized (v_max x, x, x twice) when they come out of an MFMA or a
// cross-lane move; this one is the bare instruction.  Same precondition: no NaN.
__device__ inline float max_raw(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// ---- cross-lane: combine the two 32-lane halves of a wave -------------------
// v_permlane32_swap(a, b) exchanges a[32..63] with b[0..31]: called with (x, x) it returns
// {x.lo, x.lo} and {x.hi, x.hi}, so one swap plus one ALU op reduces over the halves.
__device__ inline float xhalf_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}


// ---- phi^-1(phi(.)) of two P values with the hardware FP4 converts ------------
// v_cvt_scalef32_pk_fp4_f32 rounds to E2M1 with ties-to-even and saturates at 6 (checked
// against the threshold definition on the device, including +-3 ulp around every tie).
// r0, r1 = p * (1/s);  returns the fp16 pair (s*c0, s*c1), exact in fp16.
__device__ inline uint32_t fq_pair_f16(float r0, float r1, uint32_t s_f16x2) {
    const uint32_t codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, r0, r1, 1.0f, 0);
    const half2v c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 0);
    const half2v s = __builtin_bit_cast(half2v, s_f16x2);
    return __builtin_bit_cast(uint32_t, c * s);
}
// Eight values at once: the four converts fill one register of codes byte by byte (one
// zero-initialisation instead of four).  r[i] = p[i] * (1/s); out[j] = fp16 pair (s*c[2j], s*c[2j+1]).
__device__ inline void fq_oct_f16(const float (&r)[8], uint32_t s_f16x2, uint32_t (&out)[4]) {
    uint32_t codes = 0u;
    codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, r[0], r[1], 1.0f, 0);
    codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, r[2], r[3], 1.0f, 1);
    codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, r[4], r[5], 1.0f, 2);
    codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, r[6], r[7], 1.0f, 3);
    const half2v s = __builtin_bit_cast(half2v, s_f16x2);
    out[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 0) * s);
    out[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 1) * s);
    out[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 2) * s);
    out[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, 3) * s);
}
// The same, returning the two dequantized values as fp32 (for bf16 consumers).
__device__ inline void fq_pair_f32(float r0, float r1, float s, float& o0, float& o1) {
    typedef float float2v __attribute__((ext_vector_type(2)));
    const uint32_t codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, r0, r1, 1.0f, 0);
    const float2v c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0);
    o0 = c[0] * s; o1 = c[1] * s;
}

// ---- LDS tiles filled by direct global->LDS loads ------------------------------
// global_load_lds_dwordx4 writes lane i's 16 bytes to (wave-uniform LDS base) + 16*i, so a
// tile row cannot be padded; bank conflicts are avoided by an XOR swizzle of the 16-byte
// chunk index instead.  CH = chunks per row (16: 256-byte rows, 8: 128-byte rows).
// The 16-chunk key is row with its two 2-bit fields exchanged: 16 consecutive rows still get
// 16 distinct keys (conflict-free 16-byte column reads), and 4 consecutive rows land in 4
// different 64-byte groups (which the row-walking transpose reads below want).
template <int CH>
__device__ inline int swz(int row, int chunk) {
    return CH == 16 ? (chunk ^ (((row & 3) << 2) | ((row >> 2) & 3))) : (chunk ^ ((row >> 1) & 7));
}
// Element (row, col) of a swizzled tile with CH chunks of 8 halves per row.
template <int CH>
__device__ inline int swz_elem(int row, int col) {
    return (row * CH + swz<CH>(row, col >> 3)) * 8 + (col & 7);
}

// ds_read_b64_tr_b16: the 16 lanes of a group each pass the address of 4 consecutive 16-bit
// elements; lane i of the group receives element (i & 3) of the runs of lanes
// i/4, 4 + i/4, 8 + i/4, 12 + i/4.  With lane r pointing at X[k0 + r/4][n0 + 4*(r%4) ..],
// lane i therefore gets X[k0 .. k0+3][n0 + i]: a column of a row-major tile, i.e. the MFMA
// operand of the transposed matrix without a transposed copy.
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ inline uint2v lds_read_tr16(const uint16_t* p) {
    const short4v r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p);
    return __builtin_bit_cast(uint2v, r);
}
__device__ inline uint2v lds_read_tr16b(const unsigned char* p) { return lds_read_tr16(reinterpret_cast<const uint16_t*>(p)); }
// Plain 16-byte LDS read at a byte address.
__device__ inline uint4v lds_read16(const unsigned char* p) {
    return *(const __attribute__((address_space(3))) uint4v*)p;
}
// The same at an LDS byte address held as an integer (tiles are 256-byte aligned, so an XOR of address bits 5..7 commutes
// with adding the tile's base), and the integer address of an LDS object.
__device__ inline uint4v lds_read16_at(uint32_t addr) {
    return *(const __attribute__((address_space(3))) uint4v*)(uintptr_t)addr;
}
__device__ inline uint2v lds_read_tr16_at(uint32_t addr) {
    const short4v r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(uintptr_t)addr);
    return __builtin_bit_cast(uint2v, r);
}
__device__ inline void lds_write8_at(uint32_t addr, uint2v v) {
    *(__attribute__((address_space(3))) uint2v*)(uintptr_t)addr = v;
}
__device__ inline void lds_write16_at(uint32_t addr /* a multiple of 16 */, uint4v v) {
    *(__attribute__((address_space(3))) uint4v*)(uintptr_t)addr = v;
}
__device__ inline uint32_t lds_addr_of(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ inline uint32_t lds_read4(const unsigned char* p) {
    return *(const __attribute__((address_space(3))) uint32_t*)p;
}
// One wave copies 1 KiB: LDS chunk slot (wave-uniform slot0 + lane) <- its global source.
// Inline assembly on purpose.  The compiler files global_load_lds under FLAT accesses that may
// touch both memories, and while one is pending it turns every LDS wait of the wave into "wait
// for everything": the operand prefetch of the attention loops would drain at each product.
// Written this way the copy is invisible to the compiler's counters, so callers wait with
// s_waitcnt vmcnt(0) themselves before the barrier that publishes the tile (vector-memory
// loads return in order, so the compiler's own waits stay valid, if conservative).
// gbase: wave-uniform global address; voff: this lane's byte offset from it (< 4 GiB);
// lds_wave_base: wave-uniform LDS pointer.
__device__ inline void async_copy16(const void* gbase, uint32_t voff, void* lds_wave_base) {
    const uint32_t lds = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_wave_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(gbase), "s"(lds) : "memory");
}

// ---- workgroup -> (head, tile) with heads pinned to XCDs ----------------------
// The dispatcher hands workgroup i to XCD i % 8, and every XCD has its own L2.  All workgroups of a head stream the
// same K/V (or Q/dO) tiles, so a head is kept on one XCD: XCD x works through heads x, x + 8, ... one after another
// and its L2 sees one stream at a time instead of eight.  Needs nheads % 8 == 0 (then every XCD gets the same
// number of workgroups and the map is a bijection); otherwise the plain head-major order is kept.
__device__ inline void head_tile_of_block(int block, int nheads, int per_head, int& head, int& tile) {
    if ((nheads & 7) == 0) {
        const int xcd = block & 7, slot = block >> 3;
        head = xcd + 8 * (slot / per_head);
        tile = slot % per_head;
    } else {
        head = block / per_head;
        tile = block % per_head;
    }
}

// Host side: compute units of the current device, asked once per device (256 if the runtime does not say).
inline int device_cu_count() {
    static int ncu[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    int cus = __atomic_load_n(&ncu[dev & 63], __ATOMIC_RELAXED);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        __atomic_store_n(&ncu[dev & 63], cus, __ATOMIC_RELAXED);
    }
    return cus;
}

// Host side: raise a kernel's dynamic LDS limit once per kernel instantiation and device instead of on every launch.
// `done` is a bit mask of devices (a static of the calling instantiation).  Returns false if the runtime refuses.
inline bool ensure_dynamic_lds(const void* kernel, int bytes, unsigned long long& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const unsigned long long bit = 1ull << (dev & 63);
    if (__atomic_load_n(&done, __ATOMIC_ACQUIRE) & bit) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    __atomic_fetch_or(&done, bit, __ATOMIC_RELEASE);
    return true;
}

}  // namespace aq
