// Device-side helpers shared by the HIP kernels: storage formats and wave-level reductions (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <hip/hip_ext.h>

namespace flk {

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

// Launch with optional timing: when ev0 / ev1 are given they take the start / end time stamps of this very dispatch
// (no extra packets on the stream, so a timed launch costs what an untimed one does and the elapsed time between the two
// is the kernel's own duration); without them a plain launch.
template <typename... KArgs, typename... Args>
inline void launch_timed(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1,
                         Args... args) {
  if (ev0 || ev1) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev0, ev1, 0, static_cast<KArgs>(args)...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, st, static_cast<KArgs>(args)...);
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;   // 16 bytes of storage

template <int DT> struct Store;          // storage element of a model dtype
template <> struct Store<DT_F32> { typedef float type; };
template <> struct Store<DT_F16> { typedef uint16_t type; };
template <> struct Store<DT_BF16> { typedef uint16_t type; };

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// fp32 -> bf16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t f32_to_f16(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

template <int DT> __device__ __forceinline__ float ld(const void* p, size_t i) {
  if constexpr (DT == DT_F32) return ((const float*)p)[i];
  else if constexpr (DT == DT_F16) return f16_to_f32(((const uint16_t*)p)[i]);
  else return bf16_to_f32(((const uint16_t*)p)[i]);
}
template <int DT> __device__ __forceinline__ void st(void* p, size_t i, float v) {
  if constexpr (DT == DT_F32) ((float*)p)[i] = v;
  else if constexpr (DT == DT_F16) ((uint16_t*)p)[i] = f32_to_f16(v);
  else ((uint16_t*)p)[i] = f32_to_bf16(v);
}
// value after rounding to the model dtype
template <int DT> __device__ __forceinline__ float rdt(float v) {
  if constexpr (DT == DT_F32) return v;
  else if constexpr (DT == DT_F16) return f16_to_f32(f32_to_f16(v));
  else return bf16_to_f32(f32_to_bf16(v));
}

// 16 bytes of storage -> fp32 lanes (8 values for the 16-bit dtypes, 4 for fp32)
template <int DT> struct Vec16 { static constexpr int N = (DT == DT_F32) ? 4 : 8; };
template <int DT> __device__ __forceinline__ void unpack16(const u32x4_t& r, float* f) {
  if constexpr (DT == DT_F32) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  } else if constexpr (DT == DT_BF16) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  } else {
    f[0] = f16_to_f32((uint16_t)(r.x & 0xffffu)); f[1] = f16_to_f32((uint16_t)(r.x >> 16));
    f[2] = f16_to_f32((uint16_t)(r.y & 0xffffu)); f[3] = f16_to_f32((uint16_t)(r.y >> 16));
    f[4] = f16_to_f32((uint16_t)(r.z & 0xffffu)); f[5] = f16_to_f32((uint16_t)(r.z >> 16));
    f[6] = f16_to_f32((uint16_t)(r.w & 0xffffu)); f[7] = f16_to_f32((uint16_t)(r.w >> 16));
  }
}

// ---- layout of the 16-bit GEMM inputs (norm output, attention output, MLP activation) inside a pass
// "Fragment order": x[M][K] is kept as tiles of 16 rows x 32 k in the order the MFMA reads its row operand -- lane l
// of a tile holds x[16*mt + l%16][32*kb + 8*(l/16) .. +7] (16 bytes) -- tiles ordered [k-block][row tile], so one
// fragment load of a wave is 1 KiB contiguous and the row tiles of a k-block follow each other.  mtt = row tiles of the
// pass (ceil(M/16)); mtt == 0 means plain row-major with leading dimension ld.  k % 4 == 0 keeps 4 consecutive
// elements contiguous in both layouts.
__device__ __forceinline__ size_t xrow_index(int m, int k, int ld, int mtt) {
  if (mtt == 0) return (size_t)m * ld + k;
  return ((size_t)(k >> 5) * mtt + (m >> 4)) * 512 + ((((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7);
}

// ---- 4 consecutive elements at a time
__device__ __forceinline__ f32x4_t ld4(const float* p) { return *(const f32x4_t*)p; }
template <int DT> __device__ __forceinline__ f32x4_t ldv4(const void* p, size_t i) {   // 4 consecutive dtype elements
  if constexpr (DT == DT_F32) return *(const f32x4_t*)((const float*)p + i);
  else {
    const uint2 r = *(const uint2*)((const uint16_t*)p + i);
    if constexpr (DT == DT_BF16)
      return f32x4_t{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16),
                     __uint_as_float(r.y & 0xffff0000u)};
    else
      return f32x4_t{f16_to_f32((uint16_t)(r.x & 0xffffu)), f16_to_f32((uint16_t)(r.x >> 16)),
                     f16_to_f32((uint16_t)(r.y & 0xffffu)), f16_to_f32((uint16_t)(r.y >> 16))};
  }
}
template <int DT> __device__ __forceinline__ void stv4(void* p, size_t i, f32x4_t v) {
  if constexpr (DT == DT_F32) *(f32x4_t*)((float*)p + i) = v;
  else {
    uint2 r;
    if constexpr (DT == DT_BF16) {
      r.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
      r.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    } else {
      r.x = (uint32_t)f32_to_f16(v[0]) | ((uint32_t)f32_to_f16(v[1]) << 16);
      r.y = (uint32_t)f32_to_f16(v[2]) | ((uint32_t)f32_to_f16(v[3]) << 16);
    }
    *(uint2*)((uint16_t*)p + i) = r;
  }
}

// ---- row-wise epilogue arithmetic shared by the stand-alone kernels and the GEMM kernels that fuse them
// Floating-point contraction is switched off inside, so that the same inputs give the same bits wherever the function
// is inlined (a request's result must not depend on which variant served it).
// Rotary pair (a0, a1) = elements (i, i + d/2) of a head, (cs, sn) = cos/sin of pos * theta^(-2i/d).
__device__ __forceinline__ void rope_rotate(f32x4_t& a0, f32x4_t& a1, const f32x4_t& cs, const f32x4_t& sn) {
#pragma clang fp contract(off)
  const f32x4_t r0 = a0 * cs - a1 * sn, r1 = a1 * cs + a0 * sn;
  a0 = r0;
  a1 = r1;
}
__device__ __forceinline__ f32x4_t act_swiglu(const f32x4_t& g, const f32x4_t& u) {   // silu(g) * u
#pragma clang fp contract(off)
  f32x4_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
  return o;
}
__device__ __forceinline__ f32x4_t act_gelu(const f32x4_t& t) {                        // tanh form
#pragma clang fp contract(off)
  f32x4_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    o[e] = 0.5f * t[e] * (1.0f + tanhf(0.7978845608028654f * (t[e] + 0.044715f * t[e] * t[e] * t[e])));
  return o;
}

// ---- cross-lane: DPP within a row of 16 lanes, LDS-permute beyond.  Every step is a fixed butterfly,
// so a reduction's result does not depend on anything but the values reduced.
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
// xor-butterfly partner of `v` at distance DIST (power of two < 64); valid when all lanes at smaller distances
// already agree for DIST in {4, 8} (mirror forms), which is how the reductions below use it.
template <int DIST> __device__ __forceinline__ float partner(float v) {
  if constexpr (DIST == 1) return dpp_f<0xB1>(v);        // quad_perm [1,0,3,2]
  else if constexpr (DIST == 2) return dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
  else if constexpr (DIST == 4) return dpp_f<0x141>(v);  // row_half_mirror
  else if constexpr (DIST == 8) return dpp_f<0x140>(v);  // row_mirror
  else return __shfl_xor(v, DIST, 64);
}
// all-reduce sum over aligned groups of W lanes (W = 2..64), every lane gets the total
template <int W> __device__ __forceinline__ float group_sum(float v) {
  if constexpr (W >= 2) v += partner<1>(v);
  if constexpr (W >= 4) v += partner<2>(v);
  if constexpr (W >= 8) v += partner<4>(v);
  if constexpr (W >= 16) v += partner<8>(v);
  if constexpr (W >= 32) v += partner<16>(v);
  if constexpr (W >= 64) v += partner<32>(v);
  return v;
}
template <int W> __device__ __forceinline__ float group_max(float v) {
  if constexpr (W >= 2) v = fmaxf(v, partner<1>(v));
  if constexpr (W >= 4) v = fmaxf(v, partner<2>(v));
  if constexpr (W >= 8) v = fmaxf(v, partner<4>(v));
  if constexpr (W >= 16) v = fmaxf(v, partner<8>(v));
  if constexpr (W >= 32) v = fmaxf(v, partner<16>(v));
  if constexpr (W >= 64) v = fmaxf(v, partner<32>(v));
  return v;
}

// block-wide sum for blocks of NW waves; `red` is NW floats of LDS.  Fixed order.
template <int NW> __device__ __forceinline__ float block_sum(float v, float* red) {
  v = group_sum<64>(v);
  if constexpr (NW == 1) return v;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) t += red[i];
  return t;
}

}  // namespace flk
