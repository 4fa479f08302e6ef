// Device-side helpers shared by the HIP sources of libukv (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <type_traits>

#include "ukv_internal.h"

namespace ukv {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ void unpack8(const uint4 &w, float *f) {
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
    f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
    f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the LPR (8 or 16) adjacent lanes that share a row; every lane gets the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
    x += dpp_f<0xB1>(x);  // quad_perm [1,0,3,2]
    x += dpp_f<0x4E>(x);  // quad_perm [2,3,0,1]
    x += dpp_f<0x141>(x); // row_half_mirror
    if (LPR == 16)
        x += dpp_f<0x140>(x); // row_mirror
    return x;
}

// 128-bit load of K or V payload.  Every KV byte is used exactly once per launch, so the load
// is marked non-temporal (streaming): it keeps the L2 for page tables, q and partials.
// Pointers that reach the item functions through LDS have lost their address space; these
// casts put it back (global memory), so loads are global_load, not flat_load (which would also
// tie them to the LDS wait counter).
#define UKV_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const UKV_GLOBAL T *as_global(const T *p) {
    return (const UKV_GLOBAL T *)(p);
}
template <class T>
__device__ __forceinline__ UKV_GLOBAL T *as_global(T *p) {
    return (UKV_GLOBAL T *)(p);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4g __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_kv(const uint4 *p) {
    const u32x4 v = __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4 *>(p)));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ u32x4 ld_kv4(const void *p) {
    return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4 *>(p)));
}
// plain 128-bit global load / store
__device__ __forceinline__ uint4 ld_g16(const void *p) {
    const u32x4 v = *as_global(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_g16(float *p, float x, float y, float z, float w) {
    *as_global(reinterpret_cast<f32x4g *>(p)) = (f32x4g){x, y, z, w};
}
__device__ __forceinline__ void st_g8(float *p, float x, float y) {
    typedef float f32x2g __attribute__((ext_vector_type(2)));
    *as_global(reinterpret_cast<f32x2g *>(p)) = (f32x2g){x, y};
}
__device__ __forceinline__ u32x4 ld_g16v(const void *p) { return *as_global(reinterpret_cast<const u32x4 *>(p)); }
// 128-bit streaming store (the new token's pieces: written once, read by later launches only)
__device__ __forceinline__ void st_g16v(void *p, const u32x4 &v) {
    __builtin_nontemporal_store(v, as_global(reinterpret_cast<u32x4 *>(p)));
}
__device__ __forceinline__ void st_g16v(void *p, const uint4 &v) { st_g16v(p, (u32x4){v.x, v.y, v.z, v.w}); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Values that are the same in every lane of the workgroup, moved to scalar registers.
__device__ __forceinline__ uint32_t uni(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ uint64_t uni(uint64_t x) {
    return ((uint64_t)uni((uint32_t)(x >> 32)) << 32) | uni((uint32_t)x);
}
__device__ __forceinline__ float uni(float x) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x))); }

// Operands of the bf16 matrix instructions (v_mfma_f32_16x16x32_bf16; lane l: column l%16, k-block l/16).
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4 &w) { return __builtin_bit_cast(bf16x8_t, w); }
__device__ __forceinline__ bf16x8_t as_bf16x8(const u32x4 &w) { return __builtin_bit_cast(bf16x8_t, w); }

// Maximum over the lanes l, l^16, l^32, l^48 (the four k-blocks of one column), in every one of
// them: two lane swaps instead of two round trips through the LDS permute path.
__device__ __forceinline__ float max_over_kblocks(float x) {
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1])); // lanes [0,32) and [32,64) exchanged
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])); // odd and even rows of 16 exchanged
}

// The same for two values at once (x[0], x[1]: two blocks of columns): the first swap pairs the two values, so that the
// lower half of the wave goes on with x[0] and the upper half with x[1]; the last swap hands every lane both results.
// Three swaps and two maxima instead of four and four.
__device__ __forceinline__ void max_over_kblocks_pair(float (&x)[2]) {
    const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[0]), __float_as_uint(x[1]), false, false);
    // a[0] = (x0 of lanes < 32 | x1 of lanes < 32), a[1] = (x0 of lanes >= 32 | x1 of lanes >= 32)
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])); // lanes < 32: x0 over (l, l^32); lanes >= 32: x1
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    const float w = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])); // over (l, l^16) as well
    const auto d = __builtin_amdgcn_permlane32_swap(__float_as_uint(w), __float_as_uint(w), false, false);
    x[0] = __uint_as_float(d[0]); // (w of lanes < 32 | w of lanes < 32)
    x[1] = __uint_as_float(d[1]); // (w of lanes >= 32 | w of lanes >= 32)
}

} // namespace ukv
