// Device-side helpers shared by the Spark-FFN kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace spark {

constexpr int kWave = 64;
// cache-policy operand of the buffer loads: the nontemporal bit (data that is read once and
// should not displace what the caches hold)
constexpr int kAuxNontemporal = 2;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even; NaN stays NaN, +-inf stays +-inf (the target's own
// conversion instruction, two values at a time).
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
// (lo, hi) -> one 32-bit word holding the two bf16 values
__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
  typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
  typedef float f32x2_v __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_v{lo, hi}, bf16x2_v));
}

// One 16-byte vector of storage type T seen as VEC floats.
template <typename T>
struct Vec16;

template <>
struct Vec16<float> {
  static constexpr int N = 4;
  f32x4 raw;
  __device__ __forceinline__ float get(int i) const { return raw[i]; }
  __device__ __forceinline__ void set(int i, float v) { raw[i] = v; }
  // elements 2 i and 2 i + 1 at once
  __device__ __forceinline__ void set2(int i, float v0, float v1) {
    raw[2 * i] = v0;
    raw[2 * i + 1] = v1;
  }
  __device__ __forceinline__ static float load1(const float* p) { return *p; }
  __device__ __forceinline__ static void store1(float* p, float v) { *p = v; }
};

template <>
struct Vec16<bf16_t> {
  static constexpr int N = 8;
  u32x4 raw;
  __device__ __forceinline__ float get(int i) const {
    const uint32_t w = raw[i >> 1];
    return (i & 1) ? bf16_hi(w) : bf16_lo(w);
  }
  __device__ __forceinline__ void set(int i, float v) {
    const uint32_t h = float_to_bf16_rne(v);
    uint32_t w = raw[i >> 1];
    w = (i & 1) ? ((w & 0x0000ffffu) | (h << 16)) : ((w & 0xffff0000u) | h);
    raw[i >> 1] = w;
  }
  __device__ __forceinline__ void set2(int i, float v0, float v1) { raw[i] = pack_bf16x2_rne(v0, v1); }
  __device__ __forceinline__ static float load1(const bf16_t* p) { return bf16_bits_to_float(p->bits); }
  __device__ __forceinline__ static void store1(bf16_t* p, float v) { p->bits = float_to_bf16_rne(v); }
};

// One weight code in the OCP E4M3 format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits;
// largest finite value 448).  Rows of codes are followed, after the last row, by one fp32 scale
// per row: weight = scale * value(code).  Read-only storage type: 16 codes per 16-byte vector,
// widened by the target's conversion instruction two at a time.
struct fp8_t {
  uint8_t bits;
};
template <>
struct Vec16<fp8_t> {
  static constexpr int N = 16;
  u32x4 raw;
  __device__ __forceinline__ float get(int i) const {
    typedef float f32x2_v __attribute__((ext_vector_type(2)));
    const f32x2_v two = (i & 2) ? __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[i >> 2], true)
                                : __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[i >> 2], false);
    return two[i & 1];
  }
};

// One weight code as a signed 8-bit integer (two's complement, -127..127 used), with the same
// row layout as the E4M3 codes: weight = scale * code.
struct i8_t {
  int8_t bits;
};
template <>
struct Vec16<i8_t> {
  static constexpr int N = 16;
  u32x4 raw;
  __device__ __forceinline__ float get(int i) const {
    return (float)(int)(int8_t)(raw[i >> 2] >> (8 * (i & 3)));
  }
};

// A copy of one held vector of a packed type (bf16 pairs, 8-bit codes) that the compiler has to take
// as a new value.  A pass over vectors held in registers unpacks from such a copy (one shift, mask or
// conversion per element, and four moves per vector for the copy): without it the compiler keeps
// the widened values of one pass alive for the next, or widens vectors long before their turn,
// which multiplies the registers of a thread and lowers the rows in flight per compute unit.  The
// copies are made in program order, one vector at a time.
template <typename V>
__device__ __forceinline__ V fresh(const V& v) {
  V t = v;
  if constexpr (V::N >= 8) asm volatile("" : "+v"(t.raw));
  return t;
}

template <typename T>
__device__ __forceinline__ Vec16<T> load_vec16(const T* p) {
  Vec16<T> v;
  v.raw = *reinterpret_cast<const decltype(v.raw)*>(p);
  return v;
}

template <typename T>
__device__ __forceinline__ void store_vec16(T* p, const Vec16<T>& v) {
  *reinterpret_cast<decltype(v.raw)*>(p) = v.raw;
}

// Token vectors may be fp32 or bf16 whatever the weights are: read element i as float.
__device__ __forceinline__ float load_q(const void* q, int q_is_bf16, int64_t i) {
  return q_is_bf16 ? bf16_bits_to_float(static_cast<const uint16_t*>(q)[i])
                   : static_cast<const float*>(q)[i];
}

// N consecutive token elements starting at element i (i is a multiple of N, N = 4, 8 or 16).
template <int N>
__device__ __forceinline__ void load_q_vec(const void* q, int q_is_bf16, int64_t i, float* out) {
  if constexpr (N == 16) {
    load_q_vec<8>(q, q_is_bf16, i, out);
    load_q_vec<8>(q, q_is_bf16, i + 8, out + 8);
    return;
  }
  if (q_is_bf16) {
    const uint16_t* p = static_cast<const uint16_t*>(q) + i;
    if (N == 8) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        out[2 * e] = bf16_lo(w[e]);
        out[2 * e + 1] = bf16_hi(w[e]);
      }
    } else {
      const u32x2 w = *reinterpret_cast<const u32x2*>(p);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        out[2 * e] = bf16_lo(w[e]);
        out[2 * e + 1] = bf16_hi(w[e]);
      }
    }
  } else {
    const float* p = static_cast<const float*>(q) + i;
#pragma unroll
    for (int e = 0; e < N; e += 4) {
      const f32x4 w = *reinterpret_cast<const f32x4*>(p + e);
      out[e] = w[0];
      out[e + 1] = w[1];
      out[e + 2] = w[2];
      out[e + 3] = w[3];
    }
  }
}

// Sum over the 64 lanes of a wavefront with lane-crossing moves inside the vector unit (quad
// swaps, the two row mirrors, the two row broadcasts: no trip through the LDS crossbar); the total
// comes back as a uniform value, so every lane has it, and the order of additions is fixed, so
// the result is reproducible.
__device__ __forceinline__ float wave_sum(float v) {
  auto step = [](float x, auto ctrl, auto row_mask) {
    // lanes outside the row mask receive 0 and keep their value
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value,
                                                          decltype(row_mask)::value, 0xf, false));
  };
  v = step(v, std::integral_constant<int, 0xB1>{}, std::integral_constant<int, 0xf>{});   // quad_perm [1,0,3,2]
  v = step(v, std::integral_constant<int, 0x4E>{}, std::integral_constant<int, 0xf>{});   // quad_perm [2,3,0,1]
  v = step(v, std::integral_constant<int, 0x141>{}, std::integral_constant<int, 0xf>{});  // row_half_mirror
  v = step(v, std::integral_constant<int, 0x140>{}, std::integral_constant<int, 0xf>{});  // row_mirror
  v = step(v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});  // row_bcast:15 into rows 1 and 3
  v = step(v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});  // row_bcast:31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Number of set bits of `mask` in lanes below the calling lane.
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Sum over a thread block (THREADS a multiple of 64, <= 1024).  `red` is THREADS/64 floats
// of LDS.  All threads receive the total; the combination order is fixed.
template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float* red) {
  constexpr int NW = THREADS / kWave;
  v = wave_sum(v);
  if (NW == 1) return v;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  __syncthreads();  // protects `red` against the previous use
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += red[w];
  return t;
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_tanh(float x) {
  const float c = 0.79788456080286535588f;  // sqrt(2/pi)
  return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float gelu(float x, int kind) { return kind ? gelu_tanh(x) : gelu_erf(x); }

}  // namespace spark
