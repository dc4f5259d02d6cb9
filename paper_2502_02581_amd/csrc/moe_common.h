// Shared host/device helpers of the MoE hot-path library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/moe_hip.h"

namespace moe {

constexpr int kWave = 64;

// ---- host-side error reporting -------------------------------------------------------------
void set_error(const char* fmt, ...);
int check_shape(const moe_shape_t* s, const char* who);
bool aligned16(const void* p);
int launch_status(const char* who);

// ---- optional per-kernel timing (off by default): HIP events around every launch ------------
bool profile_on();
void profile_push(const char* label, hipStream_t st, bool begin);
struct ProfScope {
  const char* label;
  hipStream_t st;
  bool on;
  ProfScope(const char* l, hipStream_t s) : label(l), st(s), on(profile_on()) {
    if (on) profile_push(label, st, true);
  }
  ~ProfScope() {
    if (on) profile_push(label, st, false);
  }
};

// Tuning knobs: compile-time constants in the library that ships; a development build (-DMOE_TUNE)
// reads them from the environment at every launch instead, so that one build serves a sweep.
#ifdef MOE_TUNE
int tune_knob(const char* name, int dflt);
#define MOE_KNOB(name, dflt) moe::tune_knob(name, dflt)
#else
#define MOE_KNOB(name, dflt) (dflt)
#endif

inline size_t elem_size(int dtype) { return dtype == MOE_F32 ? 4 : 2; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- bf16 <-> f32 ---------------------------------------------------------------------------
typedef uint16_t bf16_t;  // storage type; arithmetic is always fp32

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Round to nearest even (NaN stays NaN) with the conversion instruction of gfx950
// (v_cvt_pk_bf16_f32: two values per instruction).  Written out with integer arithmetic and a NaN
// test, the same conversion costs a dozen instructions and a divergent branch per value, which made
// the GEMM epilogues several times slower than their stores.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  const __bf16 r = (__bf16)f;
  return __builtin_bit_cast(bf16_t, r);
}
// two values in one register: `lo` in bits 0..15
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_hw_t;
  typedef __attribute__((ext_vector_type(2))) float f32x2_hw_t;
  const f32x2_hw_t v = {lo, hi};
  const bf16x2_hw_t r = __builtin_convertvector(v, bf16x2_hw_t);
  return __builtin_bit_cast(uint32_t, r);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerVec = 4;  // elements per 16-byte vector
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPerVec = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte vector of elements widened to / narrowed from fp32
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load_nt(const float* p, float (&o)[4]) { load(p, o); }
  __device__ static __forceinline__ void load(const float* p, float (&o)[4]) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static __forceinline__ void store(float* p, const float (&o)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  // the same load with a streaming hint: for rows that nothing on the chip reads again soon
  __device__ static __forceinline__ void load_nt(const bf16_t* p, float (&o)[8]) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
#pragma unroll
    for (int i = 0; i < 4; i++) {
      o[2 * i] = __uint_as_float(v[i] << 16);
      o[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
  __device__ static __forceinline__ void load(const bf16_t* p, float (&o)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static __forceinline__ void store(bf16_t* p, const float (&o)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
      w[i] = f32x2_to_bf16x2(o[2 * i], o[2 * i + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// ---- wave-level reductions ------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}

}  // namespace moe
