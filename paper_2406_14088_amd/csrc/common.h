// Shared device/host helpers of the gfx950 generation library (no method arithmetic beyond number formats).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // storage type of a bf16 value (bit pattern): weights
typedef uint16_t f16_t;   // storage type of an IEEE half value (bit pattern): activations and KV cache

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

#define RL_WAVE 64

// bf16 -> fp32 is exact: the 16 bits are the top half of the fp32 pattern.
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Activations and the KV cache are IEEE half: 11 significant bits instead of bf16's 8, at the same
// size.  fp32 -> half rounds to nearest even and saturates at the largest finite half.
__device__ __forceinline__ f16_t f32_to_f16(float f) {
    _Float16 h = (_Float16)__builtin_amdgcn_fmed3f(f, -65504.f, 65504.f);
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    f16x2_t v = {(_Float16)__builtin_amdgcn_fmed3f(lo, -65504.f, 65504.f), (_Float16)__builtin_amdgcn_fmed3f(hi, -65504.f, 65504.f)};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float f16_to_f32(f16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ float f16lo_to_f32(uint32_t pair) { return (float)__builtin_bit_cast(f16x2_t, pair).x; }
__device__ __forceinline__ float f16hi_to_f32(uint32_t pair) { return (float)__builtin_bit_cast(f16x2_t, pair).y; }
// Two bf16 weights -> two halves.  Exact for every bf16 value whose magnitude is a normal half
// (2^-14 <= |w| <= 65504); smaller weights land on the half subnormal grid (absolute error < 2^-24).
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16lo_to_f32(w), bf16hi_to_f32(w)));
}
__device__ __forceinline__ u32x4_t bf16x8_to_f16x8(u32x4_t w) {
    u32x4_t r = {bf16x2_to_f16x2(w.x), bf16x2_to_f16x2(w.y), bf16x2_to_f16x2(w.z), bf16x2_to_f16x2(w.w)};
    return r;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Where the KV cache keeps row j of (sequence b, kv head kvh), in rows of head_dim elements from the start of a layer's
// K (or V) area.  table == NULL: contiguous slabs [max_batch][Hkv][S][hd].  Otherwise the area is a pool of pages
// [n_pages][Hkv][page][hd] with page = 1 << page_shift positions, and table[b * table_stride + (j >> page_shift)]
// names the page that holds position j of sequence b.
// kscale / vscale (both or neither): the cache rows are 16-bit block-scaled fixed point instead of IEEE half -- element e of
// row i is q[i][e] * scale[i] with q int16 and one fp32 scale per row (= per position and kv head), scale = max|x| / 32767.
// At the same 2 bytes per element a row of head_dim values of similar magnitude keeps about 15 significant bits instead of
// half's 11.  The scales of a layer's K (or V) area are indexed like its rows (kv_row_index).
struct KvMap {
    const int32_t *table = nullptr;
    int table_stride = 0;
    int page_shift = 0;
    float *kscale = nullptr;
    float *vscale = nullptr;
};
__device__ __forceinline__ size_t kv_row_index(const KvMap &m, int b, int kvh, int Hkv, int S, int j) {
    if (!m.table) return ((size_t)b * Hkv + kvh) * S + j;
    const int page = m.table[(size_t)b * m.table_stride + (j >> m.page_shift)];
    return (((size_t)page * Hkv + kvh) << m.page_shift) + (j & ((1 << m.page_shift) - 1));
}

// ---- 16-bit block-scaled rows (see KvMap)
__device__ __forceinline__ float i16lo_to_f32(uint32_t pair) { return (float)((int32_t)(pair << 16) >> 16); }
__device__ __forceinline__ float i16hi_to_f32(uint32_t pair) { return (float)((int32_t)pair >> 16); }
// inv = 32767 / max|x| of the row (0 for an all-zero row): nearest integer, kept inside +-32767
__device__ __forceinline__ int kv_quant(float x, float inv) {
    float r = rintf(x * inv);
    r = __builtin_amdgcn_fmed3f(r, -32767.f, 32767.f);
    return (int)r;
}
__device__ __forceinline__ uint32_t pack_i16x2(int lo, int hi) { return ((uint32_t)lo & 0xffffu) | ((uint32_t)hi << 16); }
__device__ __forceinline__ float kv_inv_of(float amax) { return amax > 0.f ? 32767.f / amax : 0.f; }
__device__ __forceinline__ float kv_scale_of(float amax) { return amax * (1.0f / 32767.f); }

// Two-term half split of a value: hi = half(x), lo = half(x - hi); hi + lo carries about 22 significant bits of x.
__device__ __forceinline__ uint32_t pack_f16x2_lo(float x0, float x1, uint32_t hi) {
    return pack_f16x2(x0 - f16lo_to_f32(hi), x1 - f16hi_to_f32(hi));
}

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
