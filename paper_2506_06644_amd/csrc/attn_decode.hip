// Spark-attention decode (Eq.7 of arXiv 2506.06644) for one query per head over token-major
// key / value caches (gfx950):
//
//   y = V ( softmax( Top_k^(-inf)( K1^T q[:r] ) ) * softplus( K2^T q[r:] ) )
//
// with Top_k^(-inf) the statistical top-k that sets the entries at or below
// theta = mean + std * Q(1 - k / n_ctx) to -inf (text after Eq.11).  The caches keep the
// first r entries of every key (k1c[n_ctx][r]), the rest of the key (k2c[n_ctx][d_attn - r])
// and the value (vc[n_ctx][d_attn]) in separate token-major arrays, so that the predictor
// sweep reads one dense array and everything a kept key needs is one contiguous burst per
// array (Appendix B's "row format").  Two launches for all heads of a call:
//
//   predict   s[h][g][i] = k1c_h[i] . q_hg[:r] for every cached key: a fully coalesced sweep
//             (a wave instruction covers 64 / LPR consecutive keys, LPR lanes per key); the
//             `group` query heads that share a cache are served by one pass over it.  Every
//             workgroup also leaves sum, centred sum of squares and maximum of its 256 scores.
//   gather    one workgroup per (query head): theta from the merged block statistics, then every
//             wave for itself: the kept keys among the keys it holds and, for those only, the
//             k2c and vc rows: w = exp(s - max s) * softplus(k2c[i] . q[r:]),
//             y = sum w vc[i] / sum exp(s - max s), summed in a fixed order.
//
// When n_ctx <= k every key is kept (theta = -inf); when no score exceeds theta, y = 0.
#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kKeysPerWave = 64;
constexpr int kKeysPerBlock = 4 * kKeysPerWave;   // predict: 4 waves
constexpr int kGatherWavesA = 16;    // gather: waves per workgroup
constexpr int kGatherGateCap = 512;  // keys per wave up to which the gate products have room in LDS too
constexpr int kMaxVPT = kAttnMaxCtx / (kGatherWavesA * kWave);  // scores per thread of the gather
constexpr int kStatBlocks = kAttnMaxCtx / kKeysPerBlock;         // predictor workgroups per cache at most (64)
static_assert(kStatBlocks <= kWave, "a lane per block when the gather merges the block statistics");

struct AttnParams {
  const void* k1c[kAttnMaxHeads];
  const void* k2c[kAttnMaxHeads];
  const void* vc[kAttnMaxHeads];
  const void* q;      // [heads][G][d_attn]
  float* y;           // [heads][G][d_attn]
  float* theta;       // [heads][G]         optional
  int32_t* count;     // [heads][G]         optional
  int32_t* idx;       // [heads][G][n_ctx]  optional
  float* scores;      // [heads][G][n_ctx]
  float* bstats;      // [heads][G][kStatBlocks][4]: sum, centred sum of squares and maximum of each block of 256 scores
  int n_ctx, d_attn, r, G, q_bf16, keep_all;
  float z;
};

__device__ __forceinline__ float softplus_f(float x) { return x > 0.f ? x + log1pf(expf(-x)) : log1pf(expf(x)); }

// Sum over groups of LPR consecutive lanes (LPR a power of two); every lane ends with its
// group's total.  The order of additions is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
  return x + __int_as_float(t);
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  // inside a row of 16 lanes: quad swaps and the two row mirrors (DPP, no LDS crossbar)
  if (LPR >= 2) v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  if (LPR >= 4) v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  if (LPR >= 8) v = dpp_add<0x141>(v);  // row_half_mirror
  if (LPR >= 16) v = dpp_add<0x140>(v); // row_mirror
#pragma unroll
  for (int o = 16; o < LPR; o <<= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Sums and maxima over a wavefront without the LDS crossbar (quad swaps, row mirrors, row
// broadcasts), returned as a uniform value; the order of the operations is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_other(float x) {  // lanes the row mask leaves out see their own value
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_total(float x) {
  x += dpp_other<0xB1, 0xf>(x);
  x += dpp_other<0x4E, 0xf>(x);
  x += dpp_other<0x141, 0xf>(x);
  x += dpp_other<0x140, 0xf>(x);
  // (a lane outside the row mask would add its own value: those lanes' results are not used)
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x142, 0xa, 0xf, false));
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x143, 0xc, 0xf, false));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ float wave_maximum(float x) {
  x = fmaxf(x, dpp_other<0xB1, 0xf>(x));
  x = fmaxf(x, dpp_other<0x4E, 0xf>(x));
  x = fmaxf(x, dpp_other<0x141, 0xf>(x));
  x = fmaxf(x, dpp_other<0x140, 0xf>(x));
  x = fmaxf(x, dpp_other<0x142, 0xa>(x));
  x = fmaxf(x, dpp_other<0x143, 0xc>(x));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// --------------------------------------------------------------------------------- predict
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ uint32_t raw_dword(const Vec16<bf16_t>& v, int d) { return v.raw[d]; }
__device__ __forceinline__ uint32_t raw_dword(const Vec16<float>& v, int d) { return __float_as_uint(v.raw[d]); }

// QB: bf16 caches and bf16 queries (the packed pairs go straight into the two-element dot
// product; bf16 products are exact in fp32).
template <typename WT, int LPR, int G, bool QB>
__global__ __launch_bounds__(256) void attn_predict_kernel(const AttnParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int RPI = kWave / LPR;   // keys per wave instruction
  constexpr int NI = kKeysPerWave / RPI;    // instructions per wave
  constexpr int U = NI < 16 ? NI : 16;  // loads in flight per lane
  __shared__ float s_sh[G][kKeysPerBlock];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int h = blockIdx.y, key0 = blockIdx.x * kKeysPerBlock;
  const int sub = lane / LPR, ch = lane % LPR;
  float qv[QB ? 1 : G][VEC];
  u32x4 qp[QB ? G : 1];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    if constexpr (QB) qp[g] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(P.q) + ((int64_t)h * G + g) * P.d_attn + (int64_t)ch * VEC);
    else load_q_vec<VEC>(P.q, P.q_bf16, ((int64_t)h * G + g) * P.d_attn + (int64_t)ch * VEC, qv[g]);
  }
  const WT* base = static_cast<const WT*>(P.k1c[h]);
  for (int i0 = 0; i0 < NI; i0 += U) {
    Vec16<WT> reg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = key0 + wave * kKeysPerWave + (i0 + u) * RPI + sub;
      reg[u].raw = __builtin_nontemporal_load(reinterpret_cast<const decltype(reg[u].raw)*>(
          base + (size_t)min(key, P.n_ctx - 1) * P.r + (size_t)ch * VEC));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float acc = 0.f;
        if constexpr (QB) {
#pragma unroll
          for (int d = 0; d < 4; ++d) acc = dot2_bf16(raw_dword(reg[u], d), qp[g][d], acc);
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc += reg[u].get(e) * qv[g][e];
        }
        acc = group_sum<LPR>(acc);
        if (ch == 0) s_sh[g][wave * kKeysPerWave + (i0 + u) * RPI + sub] = acc;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g)
    for (int t = tid; t < kKeysPerBlock; t += 256)
      if (key0 + t < P.n_ctx) P.scores[((size_t)h * G + g) * P.n_ctx + key0 + t] = s_sh[g][t];
  // the block's statistics (Eq.11 needs mean and standard deviation of all scores of a head: the
  // gather merges the blocks' sums and centred sums of squares): wave g serves head g
  if (wave < G) {
    const int valid = min(kKeysPerBlock, P.n_ctx - key0);
    float x[kKeysPerBlock / kWave];
    float sum = 0.f, mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kKeysPerBlock / kWave; ++i) {
      const int t = lane + kWave * i;
      x[i] = t < valid ? s_sh[wave][t] : 0.f;
      sum += x[i];
      if (t < valid) mx = fmaxf(mx, x[i]);
    }
    sum = wave_total(sum);
    mx = wave_maximum(mx);
    const float mean_b = sum / (float)valid;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kKeysPerBlock / kWave; ++i) {
      const float d = lane + kWave * i < valid ? x[i] - mean_b : 0.f;
      sq += d * d;
    }
    sq = wave_total(sq);
    if (lane == 0)
      *reinterpret_cast<f32x4*>(P.bstats + (((size_t)h * G + wave) * kStatBlocks + blockIdx.x) * 4) = f32x4{sum, sq, mx, 0.f};
  }
}

// ---------------------------------------------------------------------------------- gather
// LDS written by some lanes of a wavefront and read by others of the same wavefront
__device__ __forceinline__ void wave_lds_fence() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
}

// One workgroup of 16 waves per query head.  The workgroup forms theta and the largest score
// together (two workgroup-wide reductions); from there on every wave works alone on the kept keys
// among the keys it holds (key j = tid + T k, so the kept keys, which cluster in time, spread
// evenly over the waves): it lists them in LDS, multiplies their k2c rows by q[r:]
// (64 / LPR2 keys per step), forms the weights w = exp(s - max s) * softplus(gate) once per key
// (one lane per list position: inside the row loops the transcendentals would run for a few
// keys per instruction), and accumulates w * vc[key] (64 / LPRV keys per step; the first value
// rows are requested before the weights are formed).  The waves' rows and their sums of
// exp(s - max s) meet in LDS once, at the end, and are added in wave order.  Only a call that asks
// for the index list pays for the workgroup-wide ordered compaction.
// LDS per wave: its keys (2 bytes each), their scores (overwritten by the weights) and, when the
// context is short enough for it to fit, their gate products; with longer contexts (LEAN) the lane
// that finishes a gate product forms the weight on the spot.
// LPR2 / LPRV: lanes per k2c row / vc row (16-byte chunks).
template <typename WT, int LPR2, int LPRV>
__global__ __launch_bounds__(kGatherWavesA * kWave) void attn_gather_kernel(const AttnParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int T = kGatherWavesA * kWave;
  constexpr int KPS = kWave / LPRV;  // keys per wave step, values
  constexpr int KPG = kWave / LPR2;  // keys per wave step, gates
  static_assert(LPR2 <= LPRV, "the gate half of a key is not longer than the value");
  __shared__ float red_den[kGatherWavesA];
  __shared__ int red_cnt[kGatherWavesA];
  __shared__ int wcnt[kMaxVPT * kGatherWavesA];
  __shared__ int woff[kMaxVPT * kGatherWavesA + 1];
  extern __shared__ __align__(16) unsigned char dyn[];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int g = blockIdx.x, h = blockIdx.y, G = P.G, n = P.n_ctx;
  const int vpt = (n + T - 1) / T;    // scores per thread in use
  const int cap = vpt * kWave;        // most keys a wave can keep
  const bool lean = cap > kGatherGateCap;
  float* rows_sh = reinterpret_cast<float*>(dyn);                                   // [16][d_attn]
  float* wval = rows_sh + (size_t)kGatherWavesA * P.d_attn + (size_t)wave * cap;     // [cap] of this wave
  float* wgate = rows_sh + (size_t)kGatherWavesA * P.d_attn + (size_t)kGatherWavesA * cap + (size_t)wave * cap;  // (not LEAN)
  uint16_t* wkey = reinterpret_cast<uint16_t*>(rows_sh + (size_t)kGatherWavesA * P.d_attn + (size_t)(lean ? 1 : 2) * kGatherWavesA * cap) +
                   (size_t)wave * cap;
  const size_t hg = (size_t)h * G + g;
  const float* sc = P.scores + hg * n;

  float v[kMaxVPT];
#pragma unroll
  for (int k = 0; k < kMaxVPT; ++k) {
    const int j = tid + T * k;
    v[k] = j < n ? sc[j] : 0.f;
  }
  // theta and the largest score from the predictor's block statistics: a lane per block, every wave
  // for itself (no workgroup-wide sum): mean = sum of the sums / n, M2 = sum (M2_b + n_b (mean_b - mean)^2)
  float theta = -INFINITY, smax;
  {
    const int nblk = (n + kKeysPerBlock - 1) / kKeysPerBlock;
    const f32x4 st = lane < nblk ? *reinterpret_cast<const f32x4*>(P.bstats + (hg * kStatBlocks + lane) * 4) : f32x4{0.f, 0.f, -INFINITY, 0.f};
    const float nb = lane < nblk ? (float)min(kKeysPerBlock, n - lane * kKeysPerBlock) : 0.f;
    smax = wave_maximum(st[2]);
    if (!P.keep_all) {
      const float mean = wave_total(st[0]) / (float)n;
      const float d = lane < nblk ? st[0] / nb - mean : 0.f;
      const float m2 = wave_total(st[1] + nb * d * d);
      theta = mean + sqrtf(m2 / (float)(n - 1)) * P.z;
    }
  }

  // this wave's kept keys, in the order (k, lane) = ascending
  int nw = 0;
#pragma unroll
  for (int k = 0; k < kMaxVPT; ++k) {
    const int j = tid + T * k;
    const bool keep = j < n && v[k] > theta;
    const unsigned long long bal = __ballot(keep);
    if (keep) {
      const int pos = nw + lanes_below(bal);
      wkey[pos] = (uint16_t)j;
      wval[pos] = v[k];
    }
    if (P.idx != nullptr && lane == 0) wcnt[k * kGatherWavesA + wave] = __popcll(bal);
    nw += __popcll(bal);
  }
  if (P.idx != nullptr) {
    // the index list in ascending order over the whole workgroup: one scan over the (k, wave) counts
    __syncthreads();
    if (wave == 0) {
      int run = 0;
      for (int base = 0; base < kMaxVPT * kGatherWavesA; base += kWave) {
        const int c = wcnt[base + lane];
        int inc = c;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
          const int t = __shfl_up(inc, o, kWave);
          if (lane >= o) inc += t;
        }
        woff[base + lane] = run + inc - c;
        run += __shfl(inc, kWave - 1, kWave);
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kMaxVPT; ++k) {
      const int j = tid + T * k;
      const bool keep = j < n && v[k] > theta;
      const unsigned long long bal = __ballot(keep);
      if (keep) P.idx[hg * n + woff[k * kGatherWavesA + wave] + lanes_below(bal)] = j;
    }
  }
  wave_lds_fence();

  const int r2 = P.d_attn - P.r;
  const WT* k2 = static_cast<const WT*>(P.k2c[h]);
  const WT* vv = static_cast<const WT*>(P.vc[h]);
  const int gsub = lane / LPR2, gch = lane % LPR2;
  const int sub = lane / LPRV, ch = lane % LPRV;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  float den_mine = 0.f;
  if (nw > 0) {  // (uniform in the wave)
    float q2[VEC];
    load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)hg * P.d_attn + P.r + (int64_t)gch * VEC, q2);
    {
      constexpr int D = 4;
      auto gfetch = [&](int p, Vec16<WT>& kr) {
        const int key = wkey[min(p + gsub, nw - 1)];
        kr = load_vec16<WT>(k2 + (size_t)key * r2 + (size_t)gch * VEC);
      };
      auto guse = [&](int p, const Vec16<WT>& kr) {
        float gd = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) gd += kr.get(e) * q2[e];
        gd = group_sum<LPR2>(gd);
        if (gch == 0 && p + gsub < nw) {
          if (lean) {
            const float e0 = expf(wval[p + gsub] - smax);
            den_mine += e0;
            wval[p + gsub] = e0 * softplus_f(gd);
          } else {
            wgate[p + gsub] = gd;
          }
        }
      };
      Vec16<WT> kr[D];
#pragma unroll
      for (int d = 0; d < D; ++d) gfetch(d * KPG, kr[d]);
      for (int p = 0; p < nw; p += D * KPG) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
          guse(p + d * KPG, kr[d]);
          gfetch(p + (d + D) * KPG, kr[d]);
        }
      }
    }
    // the first value rows are requested before the weights are formed (requested together with
    // the gate rows they delay the gate products: 54 -> 57 us per step)
    constexpr int DV = 4;
    auto vfetch = [&](int p, Vec16<WT>& vr) {
      const int key = wkey[min(p + sub, nw - 1)];
      vr = load_vec16<WT>(vv + (size_t)key * P.d_attn + (size_t)ch * VEC);
    };
    Vec16<WT> vr[DV];
#pragma unroll
    for (int d = 0; d < DV; ++d) vfetch(d * KPS, vr[d]);
    wave_lds_fence();
    if (!lean) {
      for (int p = lane; p < nw; p += kWave) {
        const float e0 = expf(wval[p] - smax);
        den_mine += e0;
        wval[p] = e0 * softplus_f(wgate[p]);
      }
      wave_lds_fence();
    }
    for (int p = 0; p < nw; p += DV * KPS) {
#pragma unroll
      for (int d = 0; d < DV; ++d) {
        const int pp = p + d * KPS + sub;
        const float w = pp < nw ? wval[pp] : 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += w * vr[d].get(e);
        vfetch(p + (d + DV) * KPS, vr[d]);
      }
    }
  }
  // the lane groups of a wave, then the waves in order
#pragma unroll
  for (int o = LPRV; o < kWave; o <<= 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
  }
  const float den_wave = wave_total(den_mine);
  if (sub == 0) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) rows_sh[(size_t)wave * P.d_attn + ch * VEC + e] = acc[e];
  }
  if (lane == 0) {
    red_den[wave] = den_wave;
    red_cnt[wave] = nw;
  }
  __syncthreads();
  float den_total = 0.f;
  int count = 0;
#pragma unroll
  for (int w = 0; w < kGatherWavesA; ++w) {
    den_total += red_den[w];
    count += red_cnt[w];
  }
  if (tid == 0) {
    if (P.theta) P.theta[hg] = theta;
    if (P.count) P.count[hg] = count;
  }
  for (int c = tid; c < P.d_attn; c += T) {
    float num = 0.f;
#pragma unroll
    for (int w = 0; w < kGatherWavesA; ++w) num += rows_sh[(size_t)w * P.d_attn + c];
    P.y[hg * P.d_attn + c] = count > 0 ? num / den_total : 0.f;
  }
}

bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

template <typename WT, int LPR, bool QB>
hipError_t launch_predict_g(const AttnParams& P, dim3 grid, hipStream_t st) {
  switch (P.G) {
    case 1: hipLaunchKernelGGL((attn_predict_kernel<WT, LPR, 1, QB>), grid, dim3(256), 0, st, P); break;
    case 2: hipLaunchKernelGGL((attn_predict_kernel<WT, LPR, 2, QB>), grid, dim3(256), 0, st, P); break;
    case 3: hipLaunchKernelGGL((attn_predict_kernel<WT, LPR, 3, QB>), grid, dim3(256), 0, st, P); break;
    case 4: hipLaunchKernelGGL((attn_predict_kernel<WT, LPR, 4, QB>), grid, dim3(256), 0, st, P); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template <typename WT, bool QB>
hipError_t launch_predict_t(const AttnParams& P, int lpr, dim3 grid, hipStream_t st) {
  switch (lpr) {
    case 4: return launch_predict_g<WT, 4, QB>(P, grid, st);
    case 8: return launch_predict_g<WT, 8, QB>(P, grid, st);
    case 16: return launch_predict_g<WT, 16, QB>(P, grid, st);
    case 32: return launch_predict_g<WT, 32, QB>(P, grid, st);
    case 64: return launch_predict_g<WT, 64, QB>(P, grid, st);
    default: return hipErrorInvalidValue;
  }
}

// Dynamic LDS of the gather: the waves' rows, and per wave its keys (2 bytes), their scores / weights
// and, up to kGatherGateCap keys per wave, their gate products.
size_t gather_lds_bytes(int n_ctx, int d_attn) {
  const int T = kGatherWavesA * kWave;
  const size_t cap = (size_t)((n_ctx + T - 1) / T) * kWave;
  return (size_t)kGatherWavesA * d_attn * 4 + (size_t)kGatherWavesA * cap * ((cap > (size_t)kGatherGateCap ? 4 : 8) + 2);
}
constexpr size_t kGatherMaxLds = 150 * 1024;

template <typename WT, int LPR2, int LPRV>
hipError_t launch_gather_k(const AttnParams& P, dim3 grid, size_t dyn, hipStream_t st) {
  const void* kern = reinterpret_cast<const void*>(attn_gather_kernel<WT, LPR2, LPRV>);
  // the attribute is set to the most any call may ask for, the same value every time, so calls from
  // several threads cannot undercut each other
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGatherMaxLds);
  if (e != hipSuccess) return e;
  if (dyn > kGatherMaxLds) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_gather_kernel<WT, LPR2, LPRV>), grid, dim3(kGatherWavesA * kWave), dyn, st, P);
  return hipGetLastError();
}
template <typename WT, int LPRV>
hipError_t launch_gather_v(const AttnParams& P, int lpr2, dim3 grid, size_t dyn, hipStream_t st) {
  if constexpr (LPRV >= 4) if (lpr2 == 4) return launch_gather_k<WT, 4, LPRV>(P, grid, dyn, st);
  if constexpr (LPRV >= 8) if (lpr2 == 8) return launch_gather_k<WT, 8, LPRV>(P, grid, dyn, st);
  if constexpr (LPRV >= 16) if (lpr2 == 16) return launch_gather_k<WT, 16, LPRV>(P, grid, dyn, st);
  if constexpr (LPRV >= 32) if (lpr2 == 32) return launch_gather_k<WT, 32, LPRV>(P, grid, dyn, st);
  return hipErrorInvalidValue;
}
template <typename WT>
hipError_t launch_gather_t(const AttnParams& P, int lpr2, int lprv, dim3 grid, size_t dyn, hipStream_t st) {
  switch (lprv) {
    case 8: return launch_gather_v<WT, 8>(P, lpr2, grid, dyn, st);
    case 16: return launch_gather_v<WT, 16>(P, lpr2, grid, dyn, st);
    case 32: return launch_gather_v<WT, 32>(P, lpr2, grid, dyn, st);
    case 64: return launch_gather_v<WT, 64>(P, lpr2, grid, dyn, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool attn_supported(const AttnProblem& p) {
  const int vec = p.c_bf16 ? 8 : 4;
  if (p.r % vec || (p.d_attn - p.r) % vec || p.d_attn % vec) return false;
  const int l1 = p.r / vec, l2 = (p.d_attn - p.r) / vec, lv = p.d_attn / vec;
  return pow2(l1) && l1 >= 4 && l1 <= 64 && pow2(l2) && l2 >= 4 && pow2(lv) && lv >= 8 && lv <= 64 && l2 <= 32 &&
         p.n_ctx >= 1 && p.n_ctx <= kAttnMaxCtx && p.group >= 1 && p.group <= 4;
}

// scores [heads][group][n_ctx], then the block statistics [heads][group][kStatBlocks][4], for the
// caches of one pair of launches
size_t attn_scores_bytes(int n_heads, int group, int n_ctx) {
  const size_t per = ((size_t)group * n_ctx * 4 + 255) / 256 * 256;
  return per * (size_t)(n_heads < kAttnMaxHeads ? n_heads : kAttnMaxHeads);
}
size_t attn_workspace_bytes(int n_heads, int group, int n_ctx) {
  return attn_scores_bytes(n_heads, group, n_ctx) +
         (size_t)(n_heads < kAttnMaxHeads ? n_heads : kAttnMaxHeads) * group * kStatBlocks * 4 * sizeof(float);
}

hipError_t launch_attn_decode(const AttnProblem& p, const void* const* k1c, const void* const* k2c,
                              const void* const* vc, int n_heads, void* workspace, hipStream_t st) {
  const int vec = p.c_bf16 ? 8 : 4;
  const int l1 = p.r / vec, l2 = (p.d_attn - p.r) / vec, lv = p.d_attn / vec;
  hipError_t err = hipSuccess;
  for (int base = 0; base < n_heads && err == hipSuccess; base += kAttnMaxHeads) {
    const int H = n_heads - base < kAttnMaxHeads ? n_heads - base : kAttnMaxHeads;
    AttnParams P;
    for (int i = 0; i < kAttnMaxHeads; ++i) {
      P.k1c[i] = i < H ? k1c[base + i] : nullptr;
      P.k2c[i] = i < H ? k2c[base + i] : nullptr;
      P.vc[i] = i < H ? vc[base + i] : nullptr;
    }
    const size_t hg0 = (size_t)base * p.group;
    P.q = static_cast<const char*>(p.q) + hg0 * p.d_attn * (p.q_bf16 ? 2 : 4);
    P.y = p.y + hg0 * p.d_attn;
    P.theta = p.theta ? p.theta + hg0 : nullptr;
    P.count = p.count ? p.count + hg0 : nullptr;
    P.idx = p.idx ? p.idx + hg0 * p.n_ctx : nullptr;
    P.scores = static_cast<float*>(workspace);
    P.bstats = reinterpret_cast<float*>(static_cast<char*>(workspace) + attn_scores_bytes(n_heads, p.group, p.n_ctx));
    P.n_ctx = p.n_ctx;
    P.d_attn = p.d_attn;
    P.r = p.r;
    P.G = p.group;
    P.q_bf16 = p.q_bf16;
    P.keep_all = p.n_ctx <= p.k;
    P.z = p.z;
    const dim3 gp((p.n_ctx + kKeysPerBlock - 1) / kKeysPerBlock, H);
    if (p.c_bf16) err = p.q_bf16 ? launch_predict_t<bf16_t, true>(P, l1, gp, st) : launch_predict_t<bf16_t, false>(P, l1, gp, st);
    else err = launch_predict_t<float, false>(P, l1, gp, st);
    if (err != hipSuccess) return err;
    const size_t dyn = gather_lds_bytes(p.n_ctx, p.d_attn);
    const dim3 gg(p.group, H);
    err = p.c_bf16 ? launch_gather_t<bf16_t>(P, l2, lv, gg, dyn, st) : launch_gather_t<float>(P, l2, lv, gg, dyn, st);
  }
  return err;
}

}  // namespace spark
