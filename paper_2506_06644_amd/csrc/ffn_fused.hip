// Spark-FFN decode (Eq.2 of arXiv 2506.06644), batch 1, as ONE persistent launch over a
// stack of layers for gfx950.
//
// One workgroup per compute unit owns a contiguous slice of R = ceil(d_ff / G) neurons of
// every layer.  Inside a workgroup the wavefronts are specialised and run as a pipeline
// connected by small LDS rings, so that HBM never idles while a grid-wide dependency is
// being resolved:
//
//   stream waves   keep their share of the NEXT layer's K1n rows in flight in registers
//                  (refilled row by row as soon as a row has been consumed), compute the
//                  predictor scores s_j = K1n[j] . q[:r] and post them to an LDS ring;
//   control wave   forms the workgroup's (mean, M2) of its scores, publishes them in a
//                  16-byte slot, polls the slots of all workgroups (an all-to-all of 4 KB),
//                  merges them in a fixed order into the global mean / std, forms
//                  theta = mean + std * Q(1 - k/d_ff) (Eq.11) and the ballot mask of the
//                  workgroup's active neurons (strict s > theta), and writes the compacted
//                  ascending index list once the per-workgroup counts are known;
//   gather waves   one wavefront per active neuron: load its K2n and Vn rows (one
//                  contiguous burst each), g = K2n[j] . q[r:], u = GELU(s_j - theta) * g,
//                  accumulate u * Vn[j][:]; the waves' sums are combined in LDS in a fixed
//                  order and the workgroup's partial y is written (write-through) to a
//                  ring in the workspace, laid out so that each reader's slice is contiguous;
//   reduce wave    sums, in workgroup order, the G partials of the workgroup's own d_model/G
//                  output columns once every workgroup reports that layer as written.
//
// All cross-workgroup traffic uses agent-scope relaxed atomic loads / stores (sc1: coherent
// across the eight XCD L2s) on words that carry their own epoch, so no cache-wide
// invalidate or write-back is ever issued.  Every wait is bounded by a wall-clock timeout
// that raises an abort flag all waves observe, so the grid always drains.
//
// Results are reproducible run to run: every reduction has a fixed order.
#include <atomic>

#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kRing = 4;       // LDS ring depth (layers) for scores / theta / mask
constexpr int kPartRing = 6;   // ring depth (layers) of the partial-y buffer in the workspace
constexpr int kYRing = 3;      // LDS ring depth (layers) of the gather waves' output rows
constexpr int kReduceLag = 3;  // layers the reduce waves may trail what an exchange allowed (< kPartRing - 1)
constexpr int kRep = 8;        // replicas of the slot array (spreads the polling over channels)
constexpr int kSlotStride = 2048;  // u64 words between slot replicas (16 KB)
constexpr int kMaxG = 256;
constexpr int kSlotsPerLane = kMaxG / kWave;
constexpr size_t kProfBytes = (size_t)kMaxG * 16 * 8 * 8;  // per-wave tick counters (testing aid)
constexpr long long kTimeoutTicks = 100000000LL;  // 1 s of the 100 MHz wall clock

struct FusedParams {
  const void* k1n[kFusedMaxLayers];
  const void* k2n[kFusedMaxLayers];
  const void* vn[kFusedMaxLayers];
  const void* q;
  float* y;
  float* theta;
  int32_t* count;
  int32_t* idx;
  int32_t* ucount;
  int32_t* uidx;
  unsigned long long* slots;
  float* part;
  int32_t* status;
  long long* prof;  // optional [G][16 waves][8] tick counters (testing aid), else null
  int n_layers, d_model, d_ff, r, q_bf16, gelu;
  float z;
  int G, R, DP;  // workgroups, neurons per workgroup, d_model rounded up to 16 columns
  uint32_t epoch_base;
};

struct Shared {
  float s_ring[kRing][kWave];
  float theta_ring[kRing];
  unsigned long long mask_ring[kRing];
  int produced[kRing];  // stream-wave completions per ring slot (layer l complete at NS * (l / kRing + 1))
  int theta_ready;  // layers whose theta / mask are posted
  int g_consumed[kRing];  // gather-wave reads of a ring slot (layer l consumed at NG * (l / kRing + 1))
  int y_ready[kYRing];    // gather-wave rows posted per ybuf slot (layer l complete at NG * (l / kYRing + 1))
  int y_free;       // layers whose ybuf slot the writer wave has drained
  int p_done;       // layers whose partial row is written and acknowledged
  int r_cnt[4];     // layers finished by each reduce wave (wave i owns layers i, i + NR, ...)
  int pd_min;       // min over workgroups of layers with partial written (as last exchanged)
  int rd_min;       // min over workgroups of layers reduced (as last exchanged)
  int abort_flag;
};

__device__ __forceinline__ int lds_read(const int* p) { return *reinterpret_cast<const volatile int*>(p); }
__device__ __forceinline__ void lds_write(int* p, int v) { *reinterpret_cast<volatile int*>(p) = v; }

// LDS hand-offs between wavefronts of one workgroup: the hardware executes one wave's LDS
// operations in order, so ordering only has to be imposed on the compiler (the "memory"
// clobber) and on the return of earlier LDS loads (lgkmcnt).  Outstanding global loads
// (vmcnt) are deliberately NOT waited for: the stream waves keep theirs in flight.
__device__ __forceinline__ void lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Publishes progress: everything this wave wrote to (or read from) LDS before the call is
// ordered before the counter update.
__device__ __forceinline__ void lds_signal_add(int* p) {
  lds_fence();
  atomicAdd(p, 1);
}
__device__ __forceinline__ void lds_signal_set(int* p, int v) {
  lds_fence();
  *reinterpret_cast<volatile int*>(p) = v;
}

// Bounded wait for an LDS counter; false means the launch is being aborted.
__device__ __forceinline__ bool wait_ge(const int* p, int target, Shared* sh, int32_t* status,
                                        long long* waited = nullptr) {
  if (lds_read(p) >= target) {
    lds_fence();
    return true;
  }
  const long long tw = waited ? wall_clock64() : 0;
  long long t0 = 0;
  int spins = 0;
  while (lds_read(p) < target) {
    if (lds_read(&sh->abort_flag)) return false;
    __builtin_amdgcn_s_sleep(1);
    if ((++spins & 255) == 0) {
      const long long t = wall_clock64();
      if (t0 == 0) {
        t0 = t;
      } else if (t - t0 > kTimeoutTicks) {
        lds_write(&sh->abort_flag, 1);
        __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
      }
    }
  }
  lds_fence();
  if (waited) *waited += wall_clock64() - tw;
  return true;
}

__device__ __forceinline__ void st_u64(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_u64(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_f32(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_f32(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Raw buffer access to the ring of partial outputs: 16-byte loads / stores that bypass the
// non-coherent L2 state (sc1), addressed by a 32-bit byte offset.
constexpr int kAuxSc1 = 16;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ f32x4 buf_load_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kAuxSc1);
  return f32x4{__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3])};
}
__device__ __forceinline__ void buf_store_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 v) {
  const u32x4 u{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
  __builtin_amdgcn_raw_buffer_store_b128(u, r, (int)byte_off, 0, kAuxSc1);
}
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ int wave_min_int(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, kWave));
  return v;
}

// Sum over the wavefront with DPP moves only (no LDS crossbar): quad swaps, row mirrors, then
// the two row broadcasts; lane 63 ends with the total, which is returned as a uniform value.
// The order of additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return x + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum_dpp(float x) {
  x = dpp_add<0xB1, 0xf>(x);   // quad_perm [1,0,3,2]
  x = dpp_add<0x4E, 0xf>(x);   // quad_perm [2,3,0,1]
  x = dpp_add<0x141, 0xf>(x);  // row_half_mirror
  x = dpp_add<0x140, 0xf>(x);  // row_mirror
  x = dpp_add<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Layers reduced contiguously from 0 when reduce wave i has finished r_cnt[i] of its layers.
template <int NR>
__device__ __forceinline__ int reduced_layers(const Shared* sh) {
  int m = 1 << 30;
#pragma unroll
  for (int i = 0; i < NR; ++i) m = min(m, lds_read(&sh->r_cnt[i]) * NR + i);
  return m;
}

// Template: storage type; 16-byte chunks per lane of a K1n / K2n / Vn row; predictor rows per
// stream wave; number of stream / gather / reduce waves.
// Wave roles by index: 0 control, 1..NR reduce, NR+1 writer, then NG gather, then NS stream.
//
// Every global load below is unconditional: lanes, rows or columns that fall outside the
// problem read a valid dummy location of the same array (chunk 0 of the same row, row 0 of the
// slice, slot 0) and the value is discarded by a select.  This keeps the loads free of
// per-lane branches, so they are issued back to back and waited for only where consumed.
template <typename WT, int CPL1, int CPL2, int CPLV, int RPW, int NS, int NG, int NR>
__global__ __launch_bounds__((NS + NG + NR + 2) * kWave) void ffn_fused_kernel(const FusedParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int DM_MAX = CPLV * kWave * VEC;
  static_assert(NS * RPW <= kWave, "a workgroup owns at most 64 neurons");
  static_assert(NR >= 1 && NR <= 4, "one to four reduce waves");
  static_assert(NS + NG + NR + 2 <= 16, "at most 16 waves per workgroup");
  __shared__ Shared sh;
  __shared__ float ybuf[kYRing][NG][DM_MAX];
  __shared__ int g_has[kYRing][NG];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int w = blockIdx.x, G = P.G, R = P.R, L = P.n_layers;
  const int Rw = max(0, min(R, P.d_ff - w * R));  // neurons owned by this workgroup
  const int r2 = P.d_model - P.r;

  if (tid == 0) {
    for (int i = 0; i < kRing; ++i) sh.produced[i] = 0;
    for (int i = 0; i < 4; ++i) sh.r_cnt[i] = 0;
    for (int i = 0; i < kRing; ++i) sh.g_consumed[i] = 0;
    for (int i = 0; i < kYRing; ++i) sh.y_ready[i] = 0;
    sh.theta_ready = sh.y_free = sh.p_done = 0;
    sh.pd_min = sh.rd_min = sh.abort_flag = 0;
    if (w == 0) __hip_atomic_store(P.status, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();

  // optional tick counters of this wave: [0] lifetime, [1..7] time spent in its phases
  long long pw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const bool prof = P.prof != nullptr;
  const long long t_begin = prof ? wall_clock64() : 0;
  auto W = [&](int i) -> long long* { return prof ? &pw[i] : nullptr; };
  auto prof_flush = [&]() {
    if (prof && lane == 0) {
      pw[0] = wall_clock64() - t_begin;
      for (int i = 0; i < 8; ++i) P.prof[((size_t)w * 16 + wave) * 8 + i] = pw[i];
    }
  };

  // ------------------------------------------------------------------------------ control
  if (wave == 0) {
    unsigned long long prev_mask = 0;
    int pd_known = 0;
    for (int e = 0;; ++e) {
      const bool is_layer = e < L;
      float mean_w = 0.f, m2_w = 0.f, sval = 0.f;
      if (is_layer) {
        if (!wait_ge(&sh.produced[e % kRing], NS * (e / kRing + 1), &sh, P.status, W(1))) return;
        if (e >= kRing && !wait_ge(&sh.g_consumed[e % kRing], NG * (e / kRing), &sh, P.status, W(2))) return;
        sval = lane < Rw ? sh.s_ring[e % kRing][lane] : 0.f;
        if (Rw > 0) {
          mean_w = wave_sum_dpp(sval) / (float)Rw;
          const float dv = lane < Rw ? sval - mean_w : 0.f;
          m2_w = wave_sum_dpp(dv * dv);
        }
      }
      // The reduce waves may trail what the previous exchange allowed by at most kReduceLag
      // layers; together with kPartRing > kReduceLag + 1 this keeps the ring of partials from
      // ever blocking the exchange.
      {
        const int need = min(pd_known, L) - kReduceLag;
        if (reduced_layers<NR>(&sh) < need) {
          const long long tw = prof ? wall_clock64() : 0;
          long long t0 = 0;
          int spins = 0;
          while (reduced_layers<NR>(&sh) < need) {
            if (lds_read(&sh.abort_flag)) return;
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 255) == 0) {
              const long long t = wall_clock64();
              if (t0 == 0) {
                t0 = t;
              } else if (t - t0 > kTimeoutTicks) {
                lds_write(&sh.abort_flag, 1);
                __hip_atomic_store(P.status, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
              }
            }
          }
          if (prof) pw[3] += wall_clock64() - tw;
        }
      }
      const int cnt_prev = __popcll(prev_mask);
      const int pdone = lds_read(&sh.p_done), rdone = min(reduced_layers<NR>(&sh), L);
      const uint32_t epoch = P.epoch_base + (uint32_t)e + 1u;
      const int parity = e & 1;
      // A slot is three 64-bit words, each carrying the full epoch next to its payload, so a
      // reader can never combine words of different epochs: {mean}, {M2}, {count | pdone | rdone}.
      if (lane < kRep) {
        unsigned long long* p = P.slots + (size_t)(parity * kRep + lane) * kSlotStride + (size_t)w * 4;
        const uint32_t fields = ((uint32_t)cnt_prev << 16) | ((uint32_t)pdone << 8) | (uint32_t)rdone;
        const unsigned long long ep = (unsigned long long)epoch << 32;
        st_u64(p, ep | __float_as_uint(mean_w));
        st_u64(p + 1, ep | __float_as_uint(m2_w));
        st_u64(p + 2, ep | fields);
      }
      // poll every workgroup's slot (replica w % kRep)
      const unsigned long long* rp = P.slots + (size_t)(parity * kRep + (w % kRep)) * kSlotStride;
      unsigned long long v0[kSlotsPerLane], v1[kSlotsPerLane], v2[kSlotsPerLane];
      {
        const long long tp = prof ? wall_clock64() : 0;
        long long t0 = 0;
        int spins = 0;
        for (;;) {
#pragma unroll
          for (int i = 0; i < kSlotsPerLane; ++i) {
            const int s = lane + kWave * i;
            const unsigned long long* sp = rp + (size_t)(s < G ? s : 0) * 4;
            v0[i] = ld_u64(sp);
            v1[i] = ld_u64(sp + 1);
            v2[i] = ld_u64(sp + 2);
          }
          bool ok = true;
#pragma unroll
          for (int i = 0; i < kSlotsPerLane; ++i)
            ok = ok && ((uint32_t)(v0[i] >> 32) == epoch) && ((uint32_t)(v1[i] >> 32) == epoch) &&
                 ((uint32_t)(v2[i] >> 32) == epoch);
          if (__all(ok)) {
            if (prof) { pw[4] += wall_clock64() - tp; pw[5] += spins; }
            break;
          }
          if (lds_read(&sh.abort_flag)) return;
          if ((++spins & 63) == 0) {
            const long long t = wall_clock64();
            if (t0 == 0) {
              t0 = t;
            } else if (t - t0 > kTimeoutTicks) {
              lds_write(&sh.abort_flag, 1);
              __hip_atomic_store(P.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              return;
            }
          }
        }
      }
      // merge (Chan et al.): mean = sum n_w mean_w / n, M2 = sum M2_w + n_w (mean_w - mean)^2
      float s1 = 0.f;
      int off = 0, total = 0, pmin = 255, rmin = 255;
#pragma unroll
      for (int i = 0; i < kSlotsPerLane; ++i) {
        const int s = lane + kWave * i;
        const int nw = max(0, min(R, P.d_ff - s * R));
        const uint32_t tag = (uint32_t)v2[i];
        const int c = (tag >> 16) & 0xff;
        if (s < G) {
          s1 += (float)nw * __uint_as_float((uint32_t)v0[i]);
          off += s < w ? c : 0;
          total += c;
          pmin = min(pmin, (int)((tag >> 8) & 0xff));
          rmin = min(rmin, (int)(tag & 0xff));
        }
      }
      off = wave_sum_int(off);
      total = wave_sum_int(total);
      pmin = wave_min_int(pmin);
      rmin = wave_min_int(rmin);
      unsigned long long mask = 0;
      if (is_layer) {
        const float mean = wave_sum_dpp(s1) / (float)P.d_ff;
        float m2 = 0.f;
#pragma unroll
        for (int i = 0; i < kSlotsPerLane; ++i) {
          const int s = lane + kWave * i;
          const int nw = max(0, min(R, P.d_ff - s * R));
          if (s < G) {
            const float d = __uint_as_float((uint32_t)v0[i]) - mean;
            m2 += __uint_as_float((uint32_t)v1[i]) + (float)nw * d * d;
          }
        }
        m2 = wave_sum_dpp(m2);
        const float theta = mean + sqrtf(m2 / (float)(P.d_ff - 1)) * P.z;
        mask = __ballot(lane < Rw && sval > theta);
        if (lane == 0) {
          sh.theta_ring[e % kRing] = theta;
          sh.mask_ring[e % kRing] = mask;
          if (w == 0 && P.theta) P.theta[e] = theta;
        }
      }
      if (lane == 0) {
        lds_signal_set(&sh.pd_min, pmin);
        lds_signal_set(&sh.rd_min, rmin);
        if (is_layer) lds_signal_set(&sh.theta_ready, e + 1);
      }
      pd_known = pmin;
      // compacted index list of the previous layer: offsets are now known
      if (e >= 1 && e <= L) {
        const int layer = e - 1;
        if ((prev_mask >> lane) & 1ull) {
          const int pos = off + lanes_below(prev_mask);
          const int j = w * R + lane;
          if (P.idx) P.idx[(size_t)layer * P.d_ff + pos] = j;
          if (P.uidx) P.uidx[(size_t)layer * P.d_ff + pos] = j;
        }
        if (w == 0 && lane == 0) {
          if (P.count) P.count[layer] = total;
          if (P.ucount) P.ucount[layer] = total;
        }
      }
      prev_mask = mask;
      if (prof) pw[6] = e;
      if (!is_layer && pmin >= L) break;
      if (e > L + 4096) {
        lds_write(&sh.abort_flag, 1);
        __hip_atomic_store(P.status, 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
      }
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ reduce
  if (wave < 1 + NR) {
    // Workgroup w < DP / 16 owns output columns [16 w, 16 w + 16): one 64-byte line of every
    // workgroup's partial row.  The other workgroups have nothing to reduce.
    const int ri = wave - 1;
    const int DP = P.DP;
    const bool reader = w * 16 < DP;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(P.part, (uint32_t)kPartRing * G * DP * 4u);
    int done = 0;
    for (int l = ri; reader && l < L; l += NR) {
      if (!wait_ge(&sh.pd_min, l + 1, &sh, P.status, W(1))) return;
      const long long tl = prof ? wall_clock64() : 0;
      // every load of the layer is issued before the first use (one round trip)
      f32x4 pv[kSlotsPerLane][4];
#pragma unroll
      for (int k = 0; k < kSlotsPerLane; ++k) {
        const int t = lane + kWave * k;
        const uint32_t off = ((uint32_t)((l % kPartRing) * G + (t < G ? t : 0)) * DP + (uint32_t)w * 16u) * 4u;
#pragma unroll
        for (int i = 0; i < 4; ++i) pv[k][i] = buf_load_f32x4(prs, off + 16u * i);
      }
      float acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc[i] = 0.f;
#pragma unroll
        for (int k = 0; k < kSlotsPerLane; ++k) acc[i] += (lane + kWave * k < G) ? pv[k][i >> 2][i & 3] : 0.f;
      }
      if (prof) pw[2] += wall_clock64() - tl;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float tot = wave_sum_dpp(acc[i]);
        const int col = w * 16 + i;
        if (lane == 0 && col < P.d_model) P.y[(size_t)l * P.d_model + col] = tot;
      }
      ++done;
      if (lane == 0) lds_signal_set(&sh.r_cnt[ri], done);
      if (prof) pw[3] += wall_clock64() - tl;
    }
    // a wave that owns no further layer must not hold back the contiguous count
    if (lane == 0) lds_signal_set(&sh.r_cnt[ri], 1 << 20);
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ writer
  if (wave == 1 + NR) {
    const int DP = P.DP;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(P.part, (uint32_t)kPartRing * G * DP * 4u);
    constexpr int FPL = (DM_MAX / 4 + kWave - 1) / kWave;  // float4 columns per lane
    for (int l = 0; l < L; ++l) {
      const int ys = l % kYRing;
      if (!wait_ge(&sh.y_ready[ys], NG * (l / kYRing + 1), &sh, P.status, W(1))) return;
      // sum the gather waves' rows in wave order
      int has[NG];
#pragma unroll
      for (int g2 = 0; g2 < NG; ++g2) has[g2] = g_has[ys][g2];
      f32x4 row[FPL];
#pragma unroll
      for (int k = 0; k < FPL; ++k) {
        const int f = lane + kWave * k;
        row[k] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (f * 4 < P.d_model) {
#pragma unroll
          for (int g2 = 0; g2 < NG; ++g2)
            if (has[g2]) row[k] += *reinterpret_cast<const f32x4*>(&ybuf[ys][g2][f * 4]);
        }
      }
      lds_fence();
      if (lane == 0) lds_signal_set(&sh.y_free, l + 1);
      // the ring slot of the partial buffer must have been reduced everywhere
      if (l >= kPartRing && !wait_ge(&sh.rd_min, l - kPartRing + 1, &sh, P.status, W(2))) return;
      const long long tc = prof ? wall_clock64() : 0;
      // the workgroup's partial row, contiguous, as 16-byte write-through stores
      const uint32_t row_off = (uint32_t)((l % kPartRing) * G + w) * DP * 4u;
#pragma unroll
      for (int k = 0; k < FPL; ++k) {
        const int f = lane + kWave * k;
        if (f * 4 < DP) buf_store_f32x4(prs, row_off + (uint32_t)f * 16u, row[k]);
      }
      wait_vmem();
      if (prof) pw[3] += wall_clock64() - tc;
      if (lane == 0) lds_signal_set(&sh.p_done, l + 1);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ gather
  if (wave < 2 + NR + NG) {
    const int gw = wave - 2 - NR;
    const int nvec2 = r2 / VEC, nvecv = P.d_model / VEC;
    float q2[CPL2][VEC];
    uint32_t koff[CPL2], voff[CPLV];  // element offsets of this lane's chunks inside a row
#pragma unroll
    for (int c = 0; c < CPL2; ++c) {
      const int ch = lane + kWave * c;
      koff[c] = (uint32_t)(ch < nvec2 ? ch : 0) * VEC;
      load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)P.r + koff[c], q2[c]);
      if (ch >= nvec2) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) q2[c][e] = 0.f;
      }
    }
#pragma unroll
    for (int c = 0; c < CPLV; ++c) {
      const int ch = lane + kWave * c;
      voff[c] = (uint32_t)(ch < nvecv ? ch : 0) * VEC;
    }
    for (int l = 0; l < L; ++l) {
      if (!wait_ge(&sh.theta_ready, l + 1, &sh, P.status, W(1))) return;
      const float theta = sh.theta_ring[l % kRing];
      const unsigned long long mask_v = sh.mask_ring[l % kRing];
      const float a_lane = (lane < Rw ? sh.s_ring[l % kRing][lane] : 0.f) - theta;
      const uint32_t mlo = __builtin_amdgcn_readfirstlane((uint32_t)mask_v);
      const uint32_t mhi = __builtin_amdgcn_readfirstlane((uint32_t)(mask_v >> 32));
      unsigned long long m = ((unsigned long long)mhi << 32) | mlo;
      lds_fence();  // the ring reads above have returned
      if (lane == 0) lds_signal_add(&sh.g_consumed[l % kRing]);

      float yacc[CPLV][VEC];
#pragma unroll
      for (int c = 0; c < CPLV; ++c)
#pragma unroll
        for (int e = 0; e < VEC; ++e) yacc[c][e] = 0.f;
      int mine = 0;
      const WT* k2base = static_cast<const WT*>(P.k2n[l]);
      const WT* vbase = static_cast<const WT*>(P.vn[l]);
      const long long tn = prof ? wall_clock64() : 0;
      for (int p = 0; m != 0; ++p) {
        const int nl = __builtin_ctzll(m);
        m &= m - 1;
        if (p % NG != gw) continue;
        ++mine;
        const int64_t j = (int64_t)w * R + nl;
        const WT* k2row = k2base + j * r2;
        const WT* vrow = vbase + j * P.d_model;
        Vec16<WT> kreg[CPL2], vreg[CPLV];
#pragma unroll
        for (int c = 0; c < CPL2; ++c) kreg[c] = load_vec16<WT>(k2row + koff[c]);
#pragma unroll
        for (int c = 0; c < CPLV; ++c) vreg[c] = load_vec16<WT>(vrow + voff[c]);
        float g = 0.f;
#pragma unroll
        for (int c = 0; c < CPL2; ++c)
#pragma unroll
          for (int e = 0; e < VEC; ++e) g += kreg[c].get(e) * q2[c][e];
        g = wave_sum_dpp(g);
        const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a_lane), nl));
        const float u = gelu(a, P.gelu) * g;
#pragma unroll
        for (int c = 0; c < CPLV; ++c)
#pragma unroll
          for (int e = 0; e < VEC; ++e) yacc[c][e] += u * vreg[c].get(e);
      }
      if (prof) { pw[5] += wall_clock64() - tn; pw[6] += mine; }
      // post this wave's row to the LDS ring; the writer wave combines and stores it
      const int ys = l % kYRing;
      if (l >= kYRing && !wait_ge(&sh.y_free, l - kYRing + 1, &sh, P.status, W(2))) return;
      if (mine) {
#pragma unroll
        for (int c = 0; c < CPLV; ++c) {
          const int ch = lane + kWave * c;
          if (ch < nvecv) {
            float* dst = &ybuf[ys][gw][ch * VEC];
#pragma unroll
            for (int e = 0; e < VEC; e += 4)
              *reinterpret_cast<f32x4*>(dst + e) = f32x4{yacc[c][e], yacc[c][e + 1], yacc[c][e + 2], yacc[c][e + 3]};
          }
        }
      }
      if (lane == 0) g_has[ys][gw] = mine;
      lds_fence();
      if (lane == 0) lds_signal_add(&sh.y_ready[ys]);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ stream
  {
    const int sw = wave - 2 - NR - NG;
    const int nvec1 = P.r / VEC;
    float q1[CPL1][VEC];
    uint32_t eoff[RPW][CPL1];  // element offset of (row, chunk) inside a layer's K1n
    bool rvalid[RPW];
#pragma unroll
    for (int c = 0; c < CPL1; ++c) {
      const int ch = lane + kWave * c;
      const uint32_t co = (uint32_t)(ch < nvec1 ? ch : 0) * VEC;
      load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)co, q1[c]);
      if (ch >= nvec1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) q1[c][e] = 0.f;
      }
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        const int lr = sw + NS * i;
        const int row = (Rw > 0) ? w * R + (lr < Rw ? lr : 0) : 0;
        eoff[i][c] = (uint32_t)row * (uint32_t)P.r + co;
      }
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) rvalid[i] = sw + NS * i < Rw;

    Vec16<WT> reg[RPW][CPL1];
    {
      const WT* base0 = static_cast<const WT*>(P.k1n[0]);
#pragma unroll
      for (int i = 0; i < RPW; ++i)
#pragma unroll
        for (int c = 0; c < CPL1; ++c) reg[i][c] = load_vec16<WT>(base0 + eoff[i][c]);
    }
    for (int l = 0; l < L; ++l) {
      if (l >= kRing && !wait_ge(&sh.g_consumed[l % kRing], NG * (l / kRing), &sh, P.status, W(1))) return;
      const bool more = l + 1 < L;
      const WT* next = static_cast<const WT*>(P.k1n[more ? l + 1 : l]);
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < CPL1; ++c)
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc += reg[i][c].get(e) * q1[c][e];
        if (more) {
#pragma unroll
          for (int c = 0; c < CPL1; ++c) reg[i][c] = load_vec16<WT>(next + eoff[i][c]);
        }
        acc = wave_sum_dpp(acc);
        if (lane == 0 && rvalid[i]) sh.s_ring[l % kRing][sw + NS * i] = acc;
      }
      if (lane == 0) lds_signal_add(&sh.produced[l % kRing]);
    }
    prof_flush();
  }
}

template <typename WT, int CPL1, int CPL2, int CPLV, int RPW, int NS, int NG, int NR>
hipError_t launch_variant(const FusedParams& P, hipStream_t st) {
  auto kern = ffn_fused_kernel<WT, CPL1, CPL2, CPLV, RPW, NS, NG, NR>;
  void* args[] = {const_cast<FusedParams*>(&P)};
  return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(kern), dim3(P.G), dim3((NS + NG + NR + 2) * kWave),
                                    args, 0, st);
}

uint32_t next_epoch_base(int n_layers) {
  // Process-wide counter: every launch gets epochs no earlier launch has written into a
  // workspace, so stale slots can never be mistaken for fresh ones.
  static std::atomic<uint32_t> counter{1u};
  return counter.fetch_add((uint32_t)n_layers + 8192u);
}

int g_fused_profile = 0;

}  // namespace

void fused_set_profile(int on) { g_fused_profile = on; }
size_t fused_profile_offset(int d_model) { return fused_scratch_bytes(d_model) - kProfBytes; }
size_t fused_profile_bytes() { return kProfBytes; }

size_t fused_scratch_bytes(int d_model) {
  const size_t slots = (size_t)2 * kRep * kSlotStride * 8;
  const size_t dp = ((size_t)d_model + 15) / 16 * 16;
  const size_t part = (size_t)kPartRing * kMaxG * dp * 4;
  return 256 + slots + part + kProfBytes;
}

// Shape limits of the compiled variants: chunks per lane of a K1n / K2n / Vn row, neurons
// and output columns per workgroup.  Returns -1 when no variant fits.
int fused_variant(const FfnProblem& p) {
  const int vec = p.w_bf16 ? 8 : 4;
  const int c1 = (p.r / vec + kWave - 1) / kWave, c2 = ((p.d_model - p.r) / vec + kWave - 1) / kWave;
  const int cv = (p.d_model / vec + kWave - 1) / kWave;
  const int R = (p.d_ff + kMaxG - 1) / kMaxG;
  if (p.d_model > 16 * kMaxG) return -1;  // one 16-column slice per workgroup at most
  if (p.w_bf16) {
    if (c1 <= 2 && c2 <= 3 && cv <= 5 && R <= 36) return 0;
    if (c1 <= 3 && c2 <= 4 && cv <= 7 && R <= 56) return 1;
    return -1;
  }
  if (c1 <= 4 && c2 <= 5 && cv <= 9 && R <= 36) return 2;
  return -1;
}

bool fused_supported(const FfnProblem& p, int n_layers) {
  return p.batch == 1 && n_layers >= 1 && fused_variant(p) >= 0;
}

// layers: n_layers problems that differ only in weights and outputs' leading index.
hipError_t launch_ffn_fused(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                            const void* const* vn, int n_layers, void* scratch, hipStream_t st) {
  hipError_t err = hipSuccess;
  for (int base = 0; base < n_layers && err == hipSuccess; base += kFusedMaxLayers) {
    const int L = min(kFusedMaxLayers, n_layers - base);
    FusedParams P;
    for (int l = 0; l < L; ++l) {
      P.k1n[l] = k1n[base + l];
      P.k2n[l] = k2n[base + l];
      P.vn[l] = vn[base + l];
    }
    for (int l = L; l < kFusedMaxLayers; ++l) P.k1n[l] = P.k2n[l] = P.vn[l] = nullptr;
    P.q = p0.q;
    P.y = p0.y + (size_t)base * p0.d_model;
    P.theta = p0.theta ? p0.theta + base : nullptr;
    P.count = p0.active_count ? p0.active_count + base : nullptr;
    P.idx = p0.active_idx ? p0.active_idx + (size_t)base * p0.d_ff : nullptr;
    P.ucount = p0.union_count ? p0.union_count + base : nullptr;
    P.uidx = p0.union_idx ? p0.union_idx + (size_t)base * p0.d_ff : nullptr;
    char* s = static_cast<char*>(scratch);
    P.status = reinterpret_cast<int32_t*>(s);
    P.slots = reinterpret_cast<unsigned long long*>(s + 256);
    P.part = reinterpret_cast<float*>(s + 256 + (size_t)2 * kRep * kSlotStride * 8);
    P.prof = g_fused_profile ? reinterpret_cast<long long*>(s + fused_scratch_bytes(p0.d_model) - kProfBytes) : nullptr;
    P.n_layers = L;
    P.d_model = p0.d_model;
    P.d_ff = p0.d_ff;
    P.r = p0.r;
    P.q_bf16 = p0.q_bf16;
    P.gelu = p0.gelu;
    P.z = p0.z;
    P.G = kMaxG;
    P.R = (p0.d_ff + P.G - 1) / P.G;
    P.DP = (p0.d_model + 15) / 16 * 16;
    P.epoch_base = next_epoch_base(L);
    switch (fused_variant(p0)) {
      case 0: err = launch_variant<bf16_t, 2, 3, 5, 4, 9, 4, 1>(P, st); break;
      case 1: err = launch_variant<bf16_t, 3, 4, 7, 8, 7, 2, 1>(P, st); break;
      case 2: err = launch_variant<float, 4, 5, 9, 4, 9, 4, 1>(P, st); break;
      default: err = hipErrorInvalidValue; break;
    }
  }
  return err;
}

}  // namespace spark
