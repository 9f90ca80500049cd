// Row-wise statistical top-k (Eq.9-11 of arXiv 2506.06644) for gfx950.
//
// One workgroup owns one row (one wavefront for rows of up to 576 16-byte vectors, 4 or 16
// wavefronts for longer ones).  The row is read from HBM once into registers (striped 16-byte
// vectors, fully coalesced), the mean and the centred sum of squares are reduced with wavefront
// sums plus a small LDS combine, theta = mean + std * Q(1 - k/n) is formed, and the
// soft-thresholded row is written once.  Active indices are compacted in ascending order with
// wave ballots and an LDS prefix table.  Rows too long for the register file fall back to a
// kernel that re-reads the row for each pass.
#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

// Exclusive scan, in place, of `n` ints in LDS by the first wavefront; returns nothing,
// the grand total is left in tab[n].  Caller synchronises before and after.
__device__ __forceinline__ void wave0_exclusive_scan(int* tab, int n) {
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    int carry = 0;
    for (int base = 0; base < n; base += kWave) {
      const int i = base + lane;
      const int v = i < n ? tab[i] : 0;
      int incl = v;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int t = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += t;
      }
      if (i < n) tab[i] = carry + incl - v;
      carry += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) tab[n] = carry;
  }
}

// Huber(a; delta) / delta for a > 0 (Section 3.2, Eq.13 / Eq.14): a^2 / (2 delta) below delta,
// a - delta / 2 from there on; delta = 0 leaves a as it is (plain soft thresholding).  The
// kernels pass 1 / delta, formed once per thread (a division per element costs as much as the
// rest of the pass); it is not used when delta = 0, where no a > 0 is below delta.
__device__ __forceinline__ float huber_over_delta(float a, float delta, float inv_delta) {
  return a < delta ? 0.5f * a * a * inv_delta : a - 0.5f * delta;
}
// Its derivative in a (Appendix A.2): a / delta below delta, 1 from there on.
__device__ __forceinline__ float huber_slope(float a, float delta, float inv_delta) { return a < delta ? a * inv_delta : 1.f; }

// The thresholding pass over a row held in registers (Eq.10, or its Huber form of Section 3.2 with
// HUBER): writes y where asked and returns the thread's number of active entries; with MASKS it also
// leaves each vector's mask of active entries (for the index list and the flags).  Entries that
// are not part of the row hold -inf and are never active.  This pass is where the kernel's
// arithmetic is, and the three forms keep the plain one (no Huber term, no masks) at 5 or 6
// instructions per element.
template <bool HUBER, bool MASKS, typename T, int THREADS, int ITEMS>
__device__ __forceinline__ int threshold_pass(const Vec16<T> (&v)[ITEMS], const int (&nv)[ITEMS], float theta, float delta,
                                              float fillv, T* yr, int tid, uint32_t (&act)[ITEMS]) {
  constexpr int VEC = Vec16<T>::N;
  const float inv_delta = HUBER ? 1.f / delta : 0.f;
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int vi = i * THREADS + tid;
    const Vec16<T> xi = fresh(v[i]);
    uint32_t m = 0;
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < VEC; e += 2) {
      const float x0 = xi.get(e), x1 = xi.get(e + 1);
      const bool a0 = x0 > theta, a1 = x1 > theta;
      if (MASKS) m |= (a0 ? (1u << e) : 0u) | (a1 ? (2u << e) : 0u);
      else cnt += (a0 ? 1 : 0) + (a1 ? 1 : 0);
      const float d0 = x0 - theta, d1 = x1 - theta;
      o.set2(e / 2, a0 ? (HUBER ? huber_over_delta(d0, delta, inv_delta) : d0) : fillv,
             a1 ? (HUBER ? huber_over_delta(d1, delta, inv_delta) : d1) : fillv);
    }
    if (MASKS) {
      act[i] = m;
      cnt += __popc(m);
    }
    if (yr != nullptr && nv[i] != 0) {
      if (nv[i] == VEC) {
        __builtin_nontemporal_store(o.raw, reinterpret_cast<decltype(o.raw)*>(yr + (int64_t)vi * VEC));
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (e < nv[i]) Vec16<T>::store1(yr + (int64_t)vi * VEC + e, o.get(e));
      }
    }
  }
  return cnt;
}

template <typename T, int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void stat_topk_cached_kernel(
    const T* x, int64_t ldx, int n, float z, int fill_neg_inf, float delta, T* y, int64_t ldy,
    float* __restrict__ theta_out, int32_t* __restrict__ count_out, int32_t* __restrict__ idx_out,
    int64_t idx_cap, int32_t* __restrict__ flags, const float* __restrict__ theta_in, float* __restrict__ stats_out) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int NW = THREADS / kWave;
  __shared__ float red[NW];
  __shared__ int tab[ITEMS * NW + 1];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * ldx;
  const int nfull = n / VEC, tail = n - nfull * VEC;

  Vec16<T> v[ITEMS];
  int nv[ITEMS];  // valid elements of each held vector
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int vi = i * THREADS + tid;
    nv[i] = vi < nfull ? VEC : (vi == nfull ? tail : 0);
    if (vi < nfull) {
      // the tensor is streamed once: keep it from displacing anything in the caches
      v[i].raw = __builtin_nontemporal_load(reinterpret_cast<const decltype(v[i].raw)*>(xr + (int64_t)vi * VEC));
    } else {
      v[i].raw = (decltype(v[i].raw))(0);
      if (vi == nfull) {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (e < tail) v[i].set(e, Vec16<T>::load1(xr + (int64_t)vi * VEC + e));
      }
    }
  }

  // Sharded use (Appendix D.2): with theta_in the row's threshold is given (the statistics were
  // combined elsewhere) and only the thresholding runs; with stats_out the kernel leaves the
  // shard's mean and centred sum of squares and stops.
  float theta;
  if (theta_in != nullptr) {
    theta = theta_in[row];
  } else {
    // entries that are not part of the row were loaded as zeros: they add nothing here
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const Vec16<T> xi = fresh(v[i]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += xi.get(e);
    }
    const float mean = block_sum<THREADS>(s, red) / (float)n;

    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const Vec16<T> xi = fresh(v[i]);
      float sv = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float c = xi.get(e) - mean;
        sv += c * c;
      }
      if (nv[i] != VEC) {  // the row's last, partial vector and the vectors past it
        sv = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float c = xi.get(e) - mean;
          sv += (e < nv[i]) ? c * c : 0.f;
        }
      }
      ss += sv;
    }
    const float m2 = block_sum<THREADS>(ss, red);
    if (stats_out != nullptr) {
      if (tid == 0) {
        stats_out[2 * row] = mean;
        stats_out[2 * row + 1] = m2;
      }
      return;
    }
    theta = mean + sqrtf(m2 / (float)(n - 1)) * z;
  }
  if (tid == 0 && theta_out) theta_out[row] = theta;

  // entries that are not part of the row become -inf: never active
#pragma unroll
  for (int i = 0; i < ITEMS; ++i)
    if (nv[i] != VEC) {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (e >= nv[i]) v[i].set(e, -__builtin_inff());
    }

  const float fillv = fill_neg_inf ? -__builtin_inff() : 0.f;
  T* yr = y ? y + row * ldy : nullptr;
  uint32_t act[ITEMS];
  int cnt;
  if (delta > 0.f) cnt = threshold_pass<true, true, T, THREADS, ITEMS>(v, nv, theta, delta, fillv, yr, tid, act);
  else if (flags != nullptr || idx_out != nullptr) cnt = threshold_pass<false, true, T, THREADS, ITEMS>(v, nv, theta, delta, fillv, yr, tid, act);
  else cnt = threshold_pass<false, false, T, THREADS, ITEMS>(v, nv, theta, delta, fillv, yr, tid, act);

  if (flags) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int vi = i * THREADS + tid;
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if ((act[i] >> e) & 1u) flags[vi * VEC + e] = 1;
    }
  }

  if (idx_out) {
    int pre[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      int below = 0, total = 0;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const uint64_t b = __ballot((act[i] >> e) & 1u);
        below += lanes_below(b);
        total += __popcll(b);
      }
      pre[i] = below;
      if (lane == 0) tab[i * NW + wave] = total;
    }
    __syncthreads();
    wave0_exclusive_scan(tab, ITEMS * NW);
    __syncthreads();
    int32_t* ir = idx_out + row * idx_cap;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int vi = i * THREADS + tid;
      int pos = tab[i * NW + wave] + pre[i];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        if ((act[i] >> e) & 1u) {
          if (pos < idx_cap) ir[pos] = vi * VEC + e;
          ++pos;
        }
      }
    }
    if (tid == 0 && count_out) count_out[row] = tab[ITEMS * NW];
  } else if (count_out) {
    const float total = block_sum<THREADS>((float)cnt, red);  // exact: counts < 2^24
    if (tid == 0) count_out[row] = (int32_t)total;
  }
}

// Fallback for rows that do not fit the register file: three reads of the row.
template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void stat_topk_stream_kernel(
    const T* x, int64_t ldx, int n, float z, int fill_neg_inf, float delta, T* y, int64_t ldy,
    float* __restrict__ theta_out, int32_t* __restrict__ count_out, int32_t* __restrict__ idx_out,
    int64_t idx_cap, int32_t* __restrict__ flags, const float* __restrict__ theta_in, float* __restrict__ stats_out) {
  constexpr int NW = THREADS / kWave;
  __shared__ float red[NW];
  __shared__ int tab[NW + 1];
  __shared__ int running;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * ldx;

  float theta;
  if (theta_in != nullptr) {
    theta = theta_in[row];
  } else {
    float s = 0.f;
    for (int i = tid; i < n; i += THREADS) s += Vec16<T>::load1(xr + i);
    const float mean = block_sum<THREADS>(s, red) / (float)n;
    float ss = 0.f;
    for (int i = tid; i < n; i += THREADS) {
      const float c = Vec16<T>::load1(xr + i) - mean;
      ss += c * c;
    }
    const float m2 = block_sum<THREADS>(ss, red);
    if (stats_out != nullptr) {
      if (tid == 0) {
        stats_out[2 * row] = mean;
        stats_out[2 * row + 1] = m2;
      }
      return;
    }
    theta = mean + sqrtf(m2 / (float)(n - 1)) * z;
  }
  const float inv_delta = delta > 0.f ? 1.f / delta : 0.f;
  if (tid == 0 && theta_out) theta_out[row] = theta;
  const float fillv = fill_neg_inf ? -__builtin_inff() : 0.f;
  if (tid == 0) running = 0;
  __syncthreads();
  int cnt = 0;
  const int rounds = (n + THREADS - 1) / THREADS;
  for (int rd = 0; rd < rounds; ++rd) {
    const int i = rd * THREADS + tid;
    float xv = 0.f;
    bool a = false;
    if (i < n) {
      xv = Vec16<T>::load1(xr + i);
      a = xv > theta;
      if (y) Vec16<T>::store1(y + row * ldy + i, a ? huber_over_delta(xv - theta, delta, inv_delta) : fillv);
      if (a && flags) flags[i] = 1;
    }
    cnt += a;
    if (idx_out) {
      const uint64_t b = __ballot(a);
      if (lane == 0) tab[wave] = __popcll(b);
      __syncthreads();
      int base = running;
      for (int w = 0; w < wave; ++w) base += tab[w];
      const int pos = base + lanes_below(b);
      if (a && pos < idx_cap) idx_out[row * idx_cap + pos] = i;
      __syncthreads();
      if (tid == 0) {
        int t = running;
        for (int w = 0; w < NW; ++w) t += tab[w];
        running = t;
      }
      __syncthreads();
    }
  }
  if (count_out) {
    const float total = block_sum<THREADS>((float)cnt, red);
    if (tid == 0) count_out[row] = (int32_t)total;
  }
}

template <typename T>
hipError_t launch_stat_topk_t(const T* x, int64_t rows, int64_t n, int64_t ldx, float z, int fill, float delta,
                              T* y, int64_t ldy, float* theta, int32_t* count, int32_t* idx,
                              int64_t idx_cap, int32_t* flags, const float* theta_in, float* stats_out, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  constexpr int VEC = Vec16<T>::N;
  const int64_t nvec = (n + VEC - 1) / VEC;
  const dim3 grid((unsigned)rows);
#define SPARK_LAUNCH_CACHED(THREADS, ITEMS)                                                        \
  hipLaunchKernelGGL((stat_topk_cached_kernel<T, THREADS, ITEMS>), grid, dim3(THREADS), 0, st, x, \
                     ldx, (int)n, z, fill, delta, y, ldy, theta, count, idx, idx_cap, flags, theta_in, stats_out)
  // rows of up to 576 vectors go to one wavefront each: the two workgroup-wide sums of the statistics
  // cost a short row more than its loads (a 4.6 KB bf16 row: 23 us for 8192 rows with 256 threads per
  // row, 15 us with 64)
  if (nvec <= 64 * 1) SPARK_LAUNCH_CACHED(64, 1);
  else if (nvec <= 64 * 2) SPARK_LAUNCH_CACHED(64, 2);
  else if (nvec <= 64 * 5) SPARK_LAUNCH_CACHED(64, 5);
  else if (nvec <= 64 * 9) SPARK_LAUNCH_CACHED(64, 9);
  else if (nvec <= 256 * 5) SPARK_LAUNCH_CACHED(256, 5);
  else if (nvec <= 256 * 9) SPARK_LAUNCH_CACHED(256, 9);
  else if (nvec <= 256 * 14) SPARK_LAUNCH_CACHED(256, 14);
  else if (nvec <= 1024 * 8) SPARK_LAUNCH_CACHED(1024, 8);
  else if (sizeof(T) == 4 && nvec <= 1024 * 16) {
    // 16 vectors per lane fit the 128-VGPR budget of a 1024-thread workgroup only for fp32
    if constexpr (sizeof(T) == 4) SPARK_LAUNCH_CACHED(1024, 16);
  } else
    hipLaunchKernelGGL((stat_topk_stream_kernel<T, 1024>), grid, dim3(1024), 0, st, x, ldx, (int)n,
                       z, fill, delta, y, ldy, theta, count, idx, idx_cap, flags, theta_in, stats_out);
#undef SPARK_LAUNCH_CACHED
  return hipGetLastError();
}


// ------------------------------------------------------------------------------- backward
// gx = gy . d(Huber(StatTop_k(x); delta) / delta)/dx for one row per workgroup (chain rule
// through theta = mean + z std, Appendix A.2):
//   w_i  = gy_i * slope(x_i - theta) where x_i > theta, else 0;   G = sum_i w_i
//   gx_j = w_j - G * (1/n + z (x_j - mean) / ((n - 1) std))
// x and gy are each read once (both rows sit in registers), gx is written once.  A constant
// row (std = 0) has no active entry: G = 0 and gx = 0.
// Slope of the Huber form at a = x - theta, zero where the entry is inactive: a / delta clamped to
// [0, 1] (one multiplication whose result is clamped), which is a / delta below delta and 1 from
// there on (Appendix A.2); without the Huber term (delta = 0) the step 1[a > 0].
template <bool HUBER>
__device__ __forceinline__ float active_slope(float a, float inv_delta) {
  if (HUBER) return __builtin_amdgcn_fmed3f(a * inv_delta, 0.f, 1.f);
  return a > 0.f ? 1.f : 0.f;
}

// The two passes of the backward kernel after theta is known: G = sum of w, then gx.
template <bool HUBER, typename T, int THREADS, int ITEMS>
__device__ __forceinline__ void vjp_passes(Vec16<T> (&v)[ITEMS], Vec16<T> (&g)[ITEMS], const int (&nv)[ITEMS], int n, float z,
                                           float mean, float sd, float theta, float delta, T* or_, int tid, float* red) {
  constexpr int VEC = Vec16<T>::N;
  const float inv_delta = HUBER ? 1.f / delta : 0.f;
  float wsum = 0.f;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const Vec16<T> xv = fresh(v[i]), gv = fresh(g[i]);
#pragma unroll
    for (int e = 0; e < VEC; ++e) wsum += gv.get(e) * active_slope<HUBER>(xv.get(e) - theta, inv_delta);
  }
  const float G = block_sum<THREADS>(wsum, red);
  const float c0 = G / (float)n, c1 = sd > 0.f ? G * z / ((float)(n - 1) * sd) : 0.f;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int vi = i * THREADS + tid;
    if (nv[i] == 0) continue;
    const Vec16<T> xi = fresh(v[i]), gi = fresh(g[i]);
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < VEC; e += 2) {
      float r[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float xv = xi.get(e + h);
        const float w = gi.get(e + h) * active_slope<HUBER>(xv - theta, inv_delta);
        r[h] = w - (c0 + c1 * (xv - mean));
      }
      o.set2(e / 2, r[0], r[1]);
    }
    if (nv[i] == VEC) {
      __builtin_nontemporal_store(o.raw, reinterpret_cast<decltype(o.raw)*>(or_ + (int64_t)vi * VEC));
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (e < nv[i]) Vec16<T>::store1(or_ + (int64_t)vi * VEC + e, o.get(e));
    }
  }
}

template <typename T, int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void stat_topk_vjp_cached_kernel(const T* x, int64_t ldx, const T* gy, int64_t ldgy,
                                                                      int n, float z, float delta, T* gx, int64_t ldgx) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int NW = THREADS / kWave;
  __shared__ float red[NW];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * ldx;
  const T* gr = gy + row * ldgy;
  const int nfull = n / VEC, tail = n - nfull * VEC;

  Vec16<T> v[ITEMS], g[ITEMS];
  int nv[ITEMS];
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int vi = i * THREADS + tid;
    nv[i] = vi < nfull ? VEC : (vi == nfull ? tail : 0);
    v[i].raw = (decltype(v[i].raw))(0);
    g[i].raw = (decltype(g[i].raw))(0);
    if (vi < nfull) {
      v[i].raw = __builtin_nontemporal_load(reinterpret_cast<const decltype(v[i].raw)*>(xr + (int64_t)vi * VEC));
      g[i].raw = __builtin_nontemporal_load(reinterpret_cast<const decltype(g[i].raw)*>(gr + (int64_t)vi * VEC));
    } else if (vi == nfull) {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (e < tail) {
          v[i].set(e, Vec16<T>::load1(xr + (int64_t)vi * VEC + e));
          g[i].set(e, Vec16<T>::load1(gr + (int64_t)vi * VEC + e));
        }
    }
  }
  // entries that are not part of the row were loaded as zeros, in x and in gy: they add nothing
  // to the sum of x, and their w below is gy * slope = 0
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const Vec16<T> xi = fresh(v[i]);
#pragma unroll
    for (int e = 0; e < VEC; ++e) s += xi.get(e);
  }
  const float mean = block_sum<THREADS>(s, red) / (float)n;
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const Vec16<T> xi = fresh(v[i]);
    float sv = 0.f;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float c = xi.get(e) - mean;
      sv += c * c;
    }
    if (nv[i] != VEC) {  // the row's last, partial vector and the vectors past it
      sv = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float c = xi.get(e) - mean;
        sv += (e < nv[i]) ? c * c : 0.f;
      }
    }
    ss += sv;
  }
  const float m2 = block_sum<THREADS>(ss, red);
  const float sd = sqrtf(m2 / (float)(n - 1));
  const float theta = mean + sd * z;
  T* or_ = gx + row * ldgx;
  if (delta > 0.f) vjp_passes<true, T, THREADS, ITEMS>(v, g, nv, n, z, mean, sd, theta, delta, or_, tid, red);
  else vjp_passes<false, T, THREADS, ITEMS>(v, g, nv, n, z, mean, sd, theta, delta, or_, tid, red);
}

// Rows too long for the register file: x is read three times, gy twice.
template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void stat_topk_vjp_stream_kernel(const T* x, int64_t ldx, const T* gy, int64_t ldgy,
                                                                      int n, float z, float delta, T* gx, int64_t ldgx) {
  constexpr int NW = THREADS / kWave;
  __shared__ float red[NW];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * ldx;
  const T* gr = gy + row * ldgy;
  float s = 0.f;
  for (int i = tid; i < n; i += THREADS) s += Vec16<T>::load1(xr + i);
  const float mean = block_sum<THREADS>(s, red) / (float)n;
  float ss = 0.f;
  for (int i = tid; i < n; i += THREADS) {
    const float c = Vec16<T>::load1(xr + i) - mean;
    ss += c * c;
  }
  const float m2 = block_sum<THREADS>(ss, red);
  const float sd = sqrtf(m2 / (float)(n - 1));
  const float theta = mean + sd * z;
  const float inv_delta = delta > 0.f ? 1.f / delta : 0.f;
  float wsum = 0.f;
  for (int i = tid; i < n; i += THREADS) {
    const float a = Vec16<T>::load1(xr + i) - theta;
    if (a > 0.f) wsum += Vec16<T>::load1(gr + i) * huber_slope(a, delta, inv_delta);
  }
  const float G = block_sum<THREADS>(wsum, red);
  const float c0 = G / (float)n, c1 = sd > 0.f ? G * z / ((float)(n - 1) * sd) : 0.f;
  for (int i = tid; i < n; i += THREADS) {
    const float xv = Vec16<T>::load1(xr + i), a = xv - theta;
    const float w = a > 0.f ? Vec16<T>::load1(gr + i) * huber_slope(a, delta, inv_delta) : 0.f;
    Vec16<T>::store1(gx + row * ldgx + i, w - (c0 + c1 * (xv - mean)));
  }
}

template <typename T>
hipError_t launch_stat_topk_vjp_t(const T* x, const T* gy, int64_t rows, int64_t n, int64_t ldx, int64_t ldgy, float z,
                                  float delta, T* gx, int64_t ldgx, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  constexpr int VEC = Vec16<T>::N;
  const int64_t nvec = (n + VEC - 1) / VEC;
  const dim3 grid((unsigned)rows);
#define SPARK_LAUNCH_VJP(THREADS, ITEMS)                                                                   \
  hipLaunchKernelGGL((stat_topk_vjp_cached_kernel<T, THREADS, ITEMS>), grid, dim3(THREADS), 0, st, x, ldx, \
                     gy, ldgy, (int)n, z, delta, gx, ldgx)
  // two rows of registers per thread: more threads per row than the forward kernel uses
  if (nvec <= 256 * 1) SPARK_LAUNCH_VJP(256, 1);
  else if (nvec <= 256 * 2) SPARK_LAUNCH_VJP(256, 2);
  else if (nvec <= 256 * 4) SPARK_LAUNCH_VJP(256, 4);
  else if (nvec <= 512 * 3) SPARK_LAUNCH_VJP(512, 3);
  else if (nvec <= 512 * 5) SPARK_LAUNCH_VJP(512, 5);
  else if (nvec <= 1024 * 4) SPARK_LAUNCH_VJP(1024, 4);
  else if (sizeof(T) == 4 && nvec <= 1024 * 6) {
    if constexpr (sizeof(T) == 4) SPARK_LAUNCH_VJP(1024, 6);
  } else
    hipLaunchKernelGGL((stat_topk_vjp_stream_kernel<T, 1024>), grid, dim3(1024), 0, st, x, ldx, gy, ldgy, (int)n, z,
                       delta, gx, ldgx);
#undef SPARK_LAUNCH_VJP
  return hipGetLastError();
}

}  // namespace

hipError_t launch_stat_topk(const void* x, int dt, int64_t rows, int64_t n, int64_t ldx, float z,
                            int fill, float delta, void* y, int64_t ldy, float* theta, int32_t* count,
                            int32_t* idx, int64_t idx_cap, int32_t* flags, hipStream_t st,
                            const float* theta_in, float* stats_out) {
  if (dt == 0)
    return launch_stat_topk_t<float>(static_cast<const float*>(x), rows, n, ldx, z, fill, delta,
                                     static_cast<float*>(y), ldy, theta, count, idx, idx_cap, flags, theta_in, stats_out, st);
  return launch_stat_topk_t<bf16_t>(static_cast<const bf16_t*>(x), rows, n, ldx, z, fill, delta,
                                    static_cast<bf16_t*>(y), ldy, theta, count, idx, idx_cap, flags, theta_in, stats_out, st);
}

// Appendix D.2, global variant: the thresholds of `rows` rows from the (mean, centred sum of
// squares) pairs of their m shards, stats[s][row][2], with n_s = ns[s] entries each: the
// pairwise update of Chan et al. with every shard against the global mean,
// mean = sum n_s mean_s / N, M2 = sum (M2_s + n_s (mean_s - mean)^2), in shard order;
// theta = mean + sqrt(M2 / (N - 1)) z.  One thread per row.
constexpr int kMaxShards = 64;
struct ShardSizes {
  float n[kMaxShards];
};
__global__ __launch_bounds__(256) void combine_shard_stats_kernel(const float* __restrict__ stats, ShardSizes sizes, int m,
                                                                  int64_t rows, float n_total, float z,
                                                                  float* __restrict__ theta, float* __restrict__ mean_out,
                                                                  float* __restrict__ std_out) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= rows) return;
  float s1 = 0.f;
  for (int s = 0; s < m; ++s) s1 += sizes.n[s] * stats[((int64_t)s * rows + row) * 2];
  const float mean = s1 / n_total;
  float m2 = 0.f;
  for (int s = 0; s < m; ++s) {
    const float d = stats[((int64_t)s * rows + row) * 2] - mean;
    m2 += stats[((int64_t)s * rows + row) * 2 + 1] + sizes.n[s] * d * d;
  }
  const float sd = sqrtf(m2 / (n_total - 1.f));
  theta[row] = mean + sd * z;
  if (mean_out) mean_out[row] = mean;
  if (std_out) std_out[row] = sd;
}

hipError_t launch_combine_shard_stats(const float* stats, const int64_t* ns, int m, int64_t rows, float z, float* theta,
                                      float* mean_out, float* std_out, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  if (m < 1 || m > kMaxShards) return hipErrorInvalidValue;
  ShardSizes sizes;
  double total = 0.0;
  for (int s = 0; s < kMaxShards; ++s) {
    sizes.n[s] = s < m ? (float)ns[s] : 0.f;
    total += s < m ? (double)ns[s] : 0.0;
  }
  hipLaunchKernelGGL(combine_shard_stats_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, stats, sizes, m, rows,
                     (float)total, z, theta, mean_out, std_out);
  return hipGetLastError();
}

hipError_t launch_stat_topk_vjp(const void* x, const void* gy, int dt, int64_t rows, int64_t n, int64_t ldx,
                                int64_t ldgy, float z, float delta, void* gx, int64_t ldgx, hipStream_t st) {
  if (dt == 0)
    return launch_stat_topk_vjp_t<float>(static_cast<const float*>(x), static_cast<const float*>(gy), rows, n, ldx,
                                         ldgy, z, delta, static_cast<float*>(gx), ldgx, st);
  return launch_stat_topk_vjp_t<bf16_t>(static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(gy), rows, n, ldx,
                                        ldgy, z, delta, static_cast<bf16_t*>(gx), ldgx, st);
}

}  // namespace spark
