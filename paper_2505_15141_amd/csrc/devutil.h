// Device-side helpers shared by the kernel files (internal): storage dtype conversion, wavefront reductions, the
// bf16 hi/lo split of fp32 operands, the KV cache's value layout.
#pragma once
#include "common.h"

namespace bs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- storage dtype helpers ----------------------------------------------------------------------
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
template <typename T> __device__ __forceinline__ T from_f(float f);
template <> __device__ __forceinline__ float from_f<float>(float f) { return f; }
// float -> bf16, round to nearest even: gfx950 has the conversion in hardware (v_cvt_pk_bf16_f32, two values per
// instruction), which the compiler emits for a cast to __bf16; four integer instructions per value otherwise
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
template <> __device__ __forceinline__ uint16_t from_f<uint16_t>(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- KV cache layout --------------------------------------------------------------------------------
// Per (sequence, kv head): K is [cache_len][hd] (a key's row is contiguous: MFMA A operand of K.Q^T).
// V of a bf16 cache is stored transposed in blocks of 32 keys, [cache_len/32][hd][32], and inside a block
// the key k = 16t + 4q + e sits at slot 8q + 4t + e: lane (d, q) of the MFMA A operand of V^T.P^T then
// finds its 8 keys in one 16-byte load, in exactly the key order in which the score accumulators of
// K.Q^T hold the probabilities.  cache_len is a multiple of 32.  fp32 caches keep V as [cache_len][hd].
template <typename T> __device__ __forceinline__ size_t v_index(int key, int d, int hd);
template <> __device__ __forceinline__ size_t v_index<float>(int key, int d, int hd) { return (size_t)key * hd + d; }
template <> __device__ __forceinline__ size_t v_index<uint16_t>(int key, int d, int hd) {
    const int k = key & 31;
    const int slot = ((k & 15) >> 2) * 8 + (k >> 4) * 4 + (k & 3);
    return ((size_t)(key >> 5) * hd + d) * 32 + slot;
}

__device__ __forceinline__ uint4 ldg16(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const bf16x2_hw v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ void split8(const float v[8], uint4& hi, uint4& lo) {
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = v[e] - to_f(from_f<uint16_t>(v[e]));
    hi = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    lo = make_uint4(pack_bf16(r[0], r[1]), pack_bf16(r[2], r[3]), pack_bf16(r[4], r[5]), pack_bf16(r[6], r[7]));
}

// ---- exchange cells {float value, uint32 flag}: device-scope accesses ------------------------------------------------
// Data handed from one workgroup to another INSIDE a kernel travels in 8-byte cells that carry their own flag: one
// store, one load, no fence, and a cell is valid when its flag is the one the reader expects.  The accesses bypass the
// per-die caches (sc1), an 8-byte cell becomes visible as a whole.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
struct DevBuf { __amdgpu_buffer_rsrc_t r; };
__device__ __forceinline__ DevBuf dev_buf(const void* base) {
    DevBuf b;
    b.r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7FFFFFFF, 0x00020000);
    return b;
}
constexpr int AUX_SC1 = 16;
// two cells at cell index c (even): one 16-byte store; each 8-byte cell becomes visible as a whole
__device__ __forceinline__ void st_cells2(DevBuf b, int c, float v0, float v1, unsigned flag) {
    const u32x4 u = {__float_as_uint(v0), flag, __float_as_uint(v1), flag};
    __builtin_amdgcn_raw_buffer_store_b128(u, b.r, c * 8, 0, AUX_SC1);
}
__device__ __forceinline__ void st_cells4(DevBuf b, int c, float v0, float v1, float v2, float v3, unsigned flag) {
    st_cells2(b, c, v0, v1, flag);
    st_cells2(b, c + 2, v2, v3, flag);
}
__device__ __forceinline__ void st_cell1(DevBuf b, int c, float v, unsigned flag) {
    const u32x2 u = {__float_as_uint(v), flag};
    __builtin_amdgcn_raw_buffer_store_b64(u, b.r, c * 8, 0, AUX_SC1);
}
__device__ __forceinline__ u32x4 ld_cells2(DevBuf b, int c) { return __builtin_amdgcn_raw_buffer_load_b128(b.r, c * 8, 0, AUX_SC1); }
__device__ __forceinline__ u32x2 ld_cell1(DevBuf b, int c) { return __builtin_amdgcn_raw_buffer_load_b64(b.r, c * 8, 0, AUX_SC1); }

}  // namespace bs
