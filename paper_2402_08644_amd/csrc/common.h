// Shared device helpers for the gfx950 kernels: bf16 storage conversion, 16-lane DPP
// reductions, raw vector loads.  Wavefront size is 64 on CDNA4; nothing here is written
// for any other target.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tandem.h"

typedef uint16_t bf16_t;  // bf16 storage: upper half of an IEEE float32

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even float32 -> bf16 bits: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32, one
// instruction for two values; NaN stays NaN)
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(hw_f32x2{lo, hi}, hw_bf16x2));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// ---- DPP moves inside a row of 16 lanes -------------------------------------------------
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a DPP row; every lane of the row receives the total
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);  // row_half_mirror
  v += dpp_f32<0x140>(v);  // row_mirror
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- raw vector loads of BYTES per lane, converted to fp32 on use -----------------------
// 16 bytes of a tensor that a launch reads exactly once (cache rows, weights).  The load carries the non-temporal
// hint, so the line is not kept for reuse on its way through the caches; a plain read of a large buffer runs
// 12 % faster with it on this chip (6.7 against 6.0 TB/s).
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream16(const void* p) {
  const stream_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <int BYTES> struct Raw;
template <> struct Raw<8> {
  uint2 v;
  __device__ __forceinline__ void load(const void* p) { v = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ void load_stream(const void* p) {
    typedef uint32_t u2 __attribute__((ext_vector_type(2)));
    const u2 t = __builtin_nontemporal_load(reinterpret_cast<const u2*>(p));
    v = make_uint2(t.x, t.y);
  }
  __device__ __forceinline__ uint32_t word(int i) const { return i == 0 ? v.x : v.y; }
};
template <> struct Raw<16> {
  uint4 v;
  __device__ __forceinline__ void load(const void* p) { v = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void load_stream(const void* p) { v = ld_stream16(p); }
  __device__ __forceinline__ uint32_t word(int i) const { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
};
template <> struct Raw<32> {
  uint4 a, b;
  __device__ __forceinline__ void load(const void* p) {
    a = reinterpret_cast<const uint4*>(p)[0];
    b = reinterpret_cast<const uint4*>(p)[1];
  }
  __device__ __forceinline__ void load_stream(const void* p) {
    a = ld_stream16(p);
    b = ld_stream16(reinterpret_cast<const uint4*>(p) + 1);
  }
  __device__ __forceinline__ uint32_t word(int i) const {
    return i == 0 ? a.x : i == 1 ? a.y : i == 2 ? a.z : i == 3 ? a.w : i == 4 ? b.x : i == 5 ? b.y : i == 6 ? b.z : b.w;
  }
};

template <typename T, int N> struct Unpack;  // Raw<sizeof(T)*N> -> float[N]
template <int N> struct Unpack<float, N> {
  __device__ __forceinline__ static void run(const Raw<4 * N>& r, float* out) {
#pragma unroll
    for (int i = 0; i < N; ++i) out[i] = __uint_as_float(r.word(i));
  }
};
template <int N> struct Unpack<bf16_t, N> {
  __device__ __forceinline__ static void run(const Raw<2 * N>& r, float* out) {
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      out[2 * i] = bf16lo_to_f32(r.word(i));
      out[2 * i + 1] = bf16hi_to_f32(r.word(i));
    }
  }
};

#define TANDEM_NEG_BIG (-1.0e30f)  // finite stand-in for "no key seen yet" (keeps exp2(m - m') NaN-free)

static inline int hip_ok(hipError_t e) { return e == hipSuccess ? TANDEM_OK : TANDEM_ERR_HIP; }

// Raises a kernel's dynamic-LDS limit to `bytes` (nothing to do up to 48 KB) once per kernel and device; safe to call
// from several threads, cheap on every later call.  Returns a tandem_status.
int ensure_dynamic_lds(const void* kernel, size_t bytes);
// Compute units of the current device (looked up once per device; 0 when the runtime cannot tell).
int compute_units();
