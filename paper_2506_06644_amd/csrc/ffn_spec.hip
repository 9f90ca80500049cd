// Spark-FFN decode (Eq.2 of arXiv 2506.06644), batch 1, as ONE persistent launch over a
// stack of layers for gfx950, with the compute units split into two kinds of workgroup.
//
// A CU's vector-memory pipeline returns data in order, so a latency-critical load issued
// behind a deep prefetch stream waits for the whole stream.  The launch therefore gives the
// two halves of the method to different CUs (one workgroup per CU, 256 workgroups, GS + GG):
//
//   GS STREAM workgroups own d_ff / GS neurons each.  Their waves keep the next layer's
//     K1n rows in flight in registers (a row is re-requested for layer l+1 as soon as it has
//     been consumed for layer l), form the predictor scores s_j = K1n[j] . q[:r] and publish
//     each score, and the workgroup's (mean, M2) of its scores, as 64-bit words that carry the
//     layer's epoch.  They never wait for anybody: HBM streams at full rate throughout.
//   GG GATHER workgroups own d_ff / GG neurons each.  Two control waves (even / odd layers)
//     poll the GS statistics slots and their own scores, merge the statistics in a fixed
//     order into the global mean / std, form theta = mean + std * Q(1 - k/d_ff) (Eq.11) and
//     the ballot mask of the active neurons (strict s > theta).  Gather waves take one active
//     neuron at a time: its K2n and Vn rows (one contiguous burst each), g = K2n[j] . q[r:],
//     u = GELU(s_j - theta) * g, and add u * Vn[j][:] into the wave's own LDS row.  A writer
//     wave sums the rows in wave order and stores the workgroup's partial output; a reduce
//     wave sums the GG partials of the workgroup's own d_model / GG output columns in
//     workgroup order and writes y, and emits the compacted ascending index list.
//
// The split is a compile-time choice per shape class (128 + 128 for the Gemma-2 2B class:
// 128 CUs still stream K1n at about three quarters of the HBM rate, and the row gathers,
// which are bound by latency and not by bandwidth, need the other half of the chip to keep
// enough rows in flight).
//
// Everything that crosses workgroups is either a 64-bit word stamped with a per-launch epoch
// (written and polled with agent-scope relaxed atomics, i.e. sc1: coherent across the eight
// XCD L2s) or bulk data ordered behind such a word.  Buffers are indexed by layer, so nothing
// is reused inside a launch and the only waits are on strictly upstream progress
// (stream -> control -> gather -> writer -> reduce); every wait is bounded by a wall-clock
// timeout that raises an abort flag.  All reductions have a fixed order: results are
// reproducible bit for bit.
#include <atomic>

#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kG = 256;            // workgroups (one per CU)
constexpr int kGroup = 32;         // consecutive workgroups per placement group (4 per XCD)
constexpr int kMaxGather = 128;    // most gather workgroups any variant uses
constexpr int kLeaders = 8;        // gather workgroups that fan synchronisation words in and out
constexpr int kCell = 64;          // 64-bit words between two leaders' words (separate 512-byte cells)
constexpr int kRing = 4;           // LDS ring depth (layers)
constexpr int kTeams = 2;          // layers a gather workgroup keeps in flight
constexpr int kStatSlots = 256;    // statistics slots reserved per layer
// 64-bit mask words of a gather workgroup's neurons (GP = gather workgroups per group of 32)
constexpr int mask_words(int gp) { return gp >= 12 ? 2 : 4; }
constexpr size_t kProfBytes = (size_t)kG * 16 * 8 * 8;
constexpr long long kTimeoutTicks = 20000000LL;  // 0.2 s of the 100 MHz wall clock

struct SpecParams {
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
  unsigned long long* stats;   // [L][kStatSlots][2]  {mean | epoch}, {M2 | epoch}
  unsigned long long* scores;  // [L][d_ff]           {s_j | epoch}
  unsigned long long* gcnt;    // [L][kMaxGather]     {active count | epoch}
  unsigned long long* gdone;   // [kMaxGather]        {layers written | launch tag}
  unsigned long long* thetaw;  // [L][kLeaders][64]   {theta | epoch} in word 0 of each 512-byte cell
  unsigned long long* gdone2;  // [kLeaders][64]      {layers written by a whole group | launch tag}
  float* part;                 // [L][GG][DP]         partial outputs
  int32_t* status;
  long long* prof;
  int n_layers, d_model, d_ff, r, q_bf16, gelu;
  float z;
  int RS;   // neurons per stream workgroup
  int NPG;  // neurons per gather workgroup
  int CWG;  // output columns per reducing workgroup (multiple of 16)
  int NR;   // reducing workgroups, ceil(d_model / CWG) <= GG
  int DP;   // CWG * NR >= d_model: floats per partial row
  uint32_t epoch_base;
};

// Synchronisation words live in LDS and are accessed through pointers that carry the LDS
// address space.  (A volatile access through a generic pointer would be emitted as a FLAT
// instruction, which counts on vmcnt as well: every poll of a flag would then wait for the
// wave's outstanding global loads, i.e. for the very prefetch it is supposed to overlap.)
typedef __attribute__((address_space(3))) int lds_int_t;
__device__ __forceinline__ volatile lds_int_t* as_lds(const int* p) { return (volatile lds_int_t*)p; }
__device__ __forceinline__ int lds_read(const int* p) { return *as_lds(p); }
__device__ __forceinline__ void lds_write(int* p, int v) { *as_lds(p) = v; }

// LDS hand-offs between wavefronts of one workgroup: the hardware executes one wave's LDS
// operations in order, so ordering only has to be imposed on the compiler (the "memory"
// clobber) and on the return of earlier LDS loads (lgkmcnt).  Outstanding global loads
// (vmcnt) are deliberately NOT waited for: the stream waves keep theirs in flight.
__device__ __forceinline__ void lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void lds_signal_add(int* p) {
  lds_fence();
  __hip_atomic_fetch_add((lds_int_t*)p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_signal_set(int* p, int v) {
  lds_fence();
  *as_lds(p) = v;
}

struct Abort {
  int* flag;        // LDS
  int32_t* status;  // global
};

// Wall-clock guard for a spin loop: call every iteration; returns true when the launch must
// be abandoned (somebody raised the flag, or this wait has lasted longer than the timeout).
struct SpinGuard {
  long long t0 = 0;
  int spins = 0;
  __device__ __forceinline__ bool expired(const Abort& ab, int code) {
    if (lds_read(ab.flag)) return true;
    if ((++spins & 127) == 0) {
      const long long t = wall_clock64();
      if (t0 == 0) {
        t0 = t;
      } else if (t - t0 > kTimeoutTicks) {
        lds_write(ab.flag, 1);
        __hip_atomic_store(ab.status, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
      }
    }
    return false;
  }
};

// Bounded wait for an LDS counter; false means the launch is being aborted.  Kept inline on
// purpose: across a call the compiler can no longer count the wave's outstanding loads and
// would wait for all of them (vmcnt(0)) at the next use, defeating the prefetch.
__device__ __forceinline__ bool wait_ge(const int* p, int target, const Abort& ab, long long* waited = nullptr) {
  if (lds_read(p) < target) {
    const long long tw = waited ? wall_clock64() : 0;
    SpinGuard g;
    while (lds_read(p) < target) {
      if (g.expired(ab, 1)) return false;
      __builtin_amdgcn_s_sleep(1);
    }
    if (waited) *waited += wall_clock64() - tw;
  }
  lds_fence();
  return true;
}

__device__ __forceinline__ void st_u64(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_u64(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long pack(float v, uint32_t epoch) {
  return ((unsigned long long)epoch << 32) | __float_as_uint(v);
}
__device__ __forceinline__ uint32_t hi32(unsigned long long v) { return (uint32_t)(v >> 32); }
__device__ __forceinline__ float lo_f32(unsigned long long v) { return __uint_as_float((uint32_t)v); }

// Raw buffer access (16-byte, sc1 = coherent across XCDs) to the partial outputs.
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
// 16-byte weight load through a buffer descriptor: uniform base + uniform row offset (SGPR) +
// per-lane byte offset (VGPR); no 64-bit address arithmetic per load.
template <typename WT>
__device__ __forceinline__ Vec16<WT> buf_load_w(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off) {
  Vec16<WT> v;
  const u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)row_off, 0);
  v.raw = __builtin_bit_cast(decltype(v.raw), u);
  return v;
}
// a.lo * b.lo + a.hi * b.hi + c on packed bf16 pairs (products of bf16 values are exact in fp32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ uint32_t raw_dword(const Vec16<bf16_t>& v, int d) { return v.raw[d]; }
__device__ __forceinline__ uint32_t raw_dword(const Vec16<float>& v, int d) { return __float_as_uint(v.raw[d]); }
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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

__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

struct StreamShared {
  float s_ring[kRing][128];
  int produced[kRing];  // stream-wave completions per ring slot (layer l complete at NS * (l / kRing + 1))
  int pub_done;         // layers whose statistics have been published
};

template <int MW>
struct GatherShared {
  float theta_ring[kRing];
  unsigned long long mask_ring[kRing][MW];
  float a_ring[kRing][MW * kWave];  // s_j - theta of the workgroup's neurons
  unsigned long long mask_hist[kFusedMaxLayers][MW];
  int theta_ready;       // layers whose theta / mask / a are posted (in layer order)
  int red_seen;          // layers a reduce wave has seen written by every gather workgroup
  int g_consumed[kRing]; // gather-wave reads of a ring slot (layer l consumed at TW * (l / kRing + 1), TW = waves of a team)
  int row_full[32];      // per (gather wave, row slot): 2 * (layer posted + 1) + (the row holds data)
  int row_free[16];      // per gather wave: layers the writer has drained
  int q2_ready;          // the shared copy of q[r:] is in LDS
};

// Template: storage type; gather workgroups per placement group of 32; 16-byte chunks per lane
// of a K1n / K2n / Vn row; predictor rows per stream wave; stream waves; gather waves; LDS
// rows per gather wave (layers a gather wave may run ahead of the writer); 16-byte chunks per
// writer of a reduce slice.
//
// Every global load below is unconditional: lanes, rows or columns that fall outside the
// problem read a valid dummy location of the same array (chunk 0 of the same row, row 0,
// slot 0) and the value is discarded by a select, so loads carry no per-lane branches and
// are issued back to back.
template <typename WT, bool QB, int GP, int CPL1, int CPL2, int CPLV, int RPW, int RIF, int NS, int NGW, int RB, int CW4, bool PROF>
__global__ __launch_bounds__(1024) void ffn_spec_kernel(const SpecParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int GS = kG / kGroup * (kGroup - GP);  // stream workgroups
  constexpr int GG = kG / kGroup * GP;             // gather workgroups
  constexpr int SPL = (GS + kWave - 1) / kWave;    // statistics slots per lane of a control wave
  constexpr int WPL = (GG + kWave - 1) / kWave;    // writers per lane of a reduce wave
  constexpr int MW = mask_words(GP);
  constexpr int FPL = CPLV * VEC / 4;              // float4 columns per lane of an LDS row
  // The gather waves work in kTeams teams: team t handles the layers l = t (mod kTeams), so a
  // workgroup has kTeams layers' row gathers in flight (the gathers are bound by latency).
  constexpr int TW = NGW / kTeams;                 // waves per team
  static_assert(NGW % kTeams == 0 && kRing % kTeams == 0, "teams");
  static_assert(NS * RPW <= 128, "a stream workgroup owns at most 128 neurons");
  static_assert(NS + 1 <= 16 && NGW + 7 <= 16, "at most 16 waves per workgroup");
  static_assert(GG % kLeaders == 0 && GG / kLeaders <= kWave, "leader groups");
  static_assert(NGW * RB <= 32, "row_full slots");
  __shared__ union {
    StreamShared s;
    GatherShared<MW> g;
  } sh;
  __shared__ float q2s[CPL2 * kWave * VEC];  // q[r:] for the gather waves (zero past its end)
  __shared__ int abort_flag;
  extern __shared__ __align__(16) float rows[];  // [NGW][RB][d_model]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int w = blockIdx.x, L = P.n_layers;
  const int grp = w / kGroup, gi = w % kGroup;
  const bool is_gather = gi >= kGroup - GP;
  const Abort ab{&abort_flag, P.status};

  if (tid == 0) {
    abort_flag = 0;
    if (is_gather) {
      sh.g.theta_ready = 0;
      sh.g.red_seen = 0;
      sh.g.q2_ready = 0;
      for (int i = 0; i < kRing; ++i) sh.g.g_consumed[i] = 0;
      for (int i = 0; i < 32; ++i) sh.g.row_full[i] = 0;
      for (int i = 0; i < 16; ++i) sh.g.row_free[i] = 0;
    } else {
      for (int i = 0; i < kRing; ++i) sh.s.produced[i] = 0;
      sh.s.pub_done = 0;
    }
    if (w == 0) __hip_atomic_store(P.status, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();

  long long pw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  constexpr bool prof = PROF;  // compiled out of the production kernels
  const long long t_begin = prof ? wall_clock64() : 0;
  auto W = [&](int i) -> long long* { return prof ? &pw[i] : nullptr; };
  auto prof_flush = [&]() {
    if (prof && lane == 0) {
      pw[0] = wall_clock64() - t_begin;
      for (int i = 0; i < 8; ++i) P.prof[((size_t)w * 16 + wave) * 8 + i] = pw[i];
    }
  };

  // profiling only: absolute time at which this wave finished layer 0 / the middle layer
  auto mark = [&](int l) {
    if (prof && l == 0) pw[6] = wall_clock64();
    if (prof && l == L - 1) pw[7] = wall_clock64();
  };

  if (!is_gather) {
    // ============================================================== STREAM workgroup
    const int s = grp * (kGroup - GP) + gi;             // index among stream workgroups
    const int RS = P.RS;
    const int RSw = max(0, min(RS, P.d_ff - s * RS));    // neurons owned
    if (wave < NS) {
      const int sw = wave;
      const int nvec1 = P.r / VEC;
      // q[:r]: as fp32, or (bf16 weights and a bf16 token) as the packed bf16 pairs themselves,
      // which the two-element dot product instruction consumes directly
      constexpr bool DOT2 = QB && VEC == 8;
      float q1[DOT2 ? 1 : CPL1][VEC];
      u32x4 q1p[DOT2 ? CPL1 : 1];
      uint32_t loff[CPL1];  // byte offset of this lane's chunks inside a row (VGPR)
      uint32_t roff[RPW];   // byte offset of the wave's rows inside a layer's K1n (SGPR)
#pragma unroll
      for (int c = 0; c < CPL1; ++c) {
        const int ch = lane + kWave * c;
        const uint32_t co = (uint32_t)(ch < nvec1 ? ch : 0) * VEC;
        if constexpr (DOT2) {
          q1p[c] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(P.q) + co);
          if (ch >= nvec1) q1p[c] = u32x4{0u, 0u, 0u, 0u};
        } else {
          load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)co, q1[c]);
          if (ch >= nvec1) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) q1[c][e] = 0.f;
          }
        }
        loff[c] = co * (uint32_t)sizeof(WT);
      }
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        const int lr = sw + NS * i;
        const int row = (RSw > 0) ? s * RS + (lr < RSw ? lr : 0) : 0;
        roff[i] = __builtin_amdgcn_readfirstlane((uint32_t)row * (uint32_t)P.r * (uint32_t)sizeof(WT));
      }

      const uint32_t k1_bytes = (uint32_t)P.d_ff * (uint32_t)P.r * (uint32_t)sizeof(WT);
      // The wave keeps RIF of its RPW rows in flight: row n + RIF (counting across layers) is
      // requested right after row n has been consumed.  The depth is a trade: enough bytes in
      // flight to cover the memory latency at full rate, but no more, because everything
      // beyond that only queues in front of the gather workgroups' latency-bound loads.
      static_assert(RIF >= 1 && RIF <= RPW, "rows in flight");
      Vec16<WT> reg[RPW][CPL1];
      {
        const __amdgpu_buffer_rsrc_t b0 = make_rsrc(P.k1n[0], k1_bytes);
#pragma unroll
        for (int i = 0; i < RIF; ++i) {
#pragma unroll
          for (int c = 0; c < CPL1; ++c) reg[i][c] = buf_load_w<WT>(b0, loff[c], roff[i]);
          // Rows are requested in the order in which they are consumed, here and in the loop:
          // the wait before a row's use then only has to cover that row's own loads.
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      for (int l = 0; l < L; ++l) {
        if (l >= kRing && !wait_ge(&sh.s.pub_done, l - kRing + 1, ab, W(1))) return;
        // After the last layer the descriptor has zero records: the loads are still issued
        // (so the number of loads in flight stays a compile-time constant and the waits can
        // be exact) but return zeros without touching memory.
        const bool more = l + 1 < L;
        const __amdgpu_buffer_rsrc_t cur = make_rsrc(P.k1n[l], k1_bytes);
        const __amdgpu_buffer_rsrc_t next = make_rsrc(P.k1n[more ? l + 1 : l], more ? k1_bytes : 0u);
        float mys = 0.f;  // lane i keeps the score of the wave's i-th row
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
          float acc = 0.f;
          if constexpr (DOT2) {
            // one accumulator per chunk: independent dependency chains
            float accc[CPL1];
#pragma unroll
            for (int c = 0; c < CPL1; ++c) {
              accc[c] = 0.f;
#pragma unroll
              for (int d = 0; d < 4; ++d) accc[c] = dot2_bf16(raw_dword(reg[i][c], d), q1p[c][d], accc[c]);
            }
#pragma unroll
            for (int c = 0; c < CPL1; ++c) acc += accc[c];
          } else {
#pragma unroll
            for (int c = 0; c < CPL1; ++c)
#pragma unroll
              for (int e = 0; e < VEC; ++e) acc += reg[i][c].get(e) * q1[c][e];
          }
          if (i + RIF < RPW) {
#pragma unroll
            for (int c = 0; c < CPL1; ++c) reg[(i + RIF) % RPW][c] = buf_load_w<WT>(cur, loff[c], roff[(i + RIF) % RPW]);
          } else {
#pragma unroll
            for (int c = 0; c < CPL1; ++c) reg[(i + RIF) % RPW][c] = buf_load_w<WT>(next, loff[c], roff[(i + RIF) % RPW]);
          }
          acc = wave_sum_dpp(acc);
          mys = lane == i ? acc : mys;
          __builtin_amdgcn_sched_barrier(0);
        }
        // Scores go to LDS only.  The publisher wave stores them to memory: a store issued
        // here would sit between this wave's loads, and since the memory counter retires in
        // order, every later load would also wait for the store's (slow, device-scope)
        // acknowledgement.
        if (lane < RPW && sw + NS * lane < RSw) sh.s.s_ring[l % kRing][sw + NS * lane] = mys;
        if (lane == 0) lds_signal_add(&sh.s.produced[l % kRing]);
        mark(l);
      }
      prof_flush();
    } else if (wave == NS) {
      // publisher: the workgroup's (mean, M2) of each layer's scores
      for (int l = 0; l < L; ++l) {
        if (!wait_ge(&sh.s.produced[l % kRing], NS * (l / kRing + 1), ab, W(1))) return;
        const float v0 = lane < RSw ? sh.s.s_ring[l % kRing][lane] : 0.f;
        const float v1 = lane + kWave < RSw ? sh.s.s_ring[l % kRing][lane + kWave] : 0.f;
        float mean_w = 0.f, m2_w = 0.f;
        if (RSw > 0) {
          mean_w = wave_sum_dpp(v0 + v1) / (float)RSw;
          const float d0 = lane < RSw ? v0 - mean_w : 0.f;
          const float d1 = lane + kWave < RSw ? v1 - mean_w : 0.f;
          m2_w = wave_sum_dpp(d0 * d0 + d1 * d1);
        }
        const uint32_t epoch = P.epoch_base + (uint32_t)l + 1u;
        unsigned long long* srow = P.scores + (size_t)l * P.d_ff + (size_t)s * RS;
        if (lane < RSw) st_u64(srow + lane, pack(v0, epoch));
        if (lane + kWave < RSw) st_u64(srow + lane + kWave, pack(v1, epoch));
        if (lane == 0) {
          unsigned long long* p = P.stats + ((size_t)l * kStatSlots + s) * 2;
          st_u64(p, pack(mean_w, epoch));
          st_u64(p + 1, pack(m2_w, epoch));
          lds_signal_set(&sh.s.pub_done, l + 1);
        }
        mark(l);
      }
      prof_flush();
    }
    return;
  }

  // ================================================================ GATHER workgroup
  const int g = grp * GP + (gi - (kGroup - GP));  // index among gather workgroups
  const int NPG = P.NPG;
  const int NPGg = max(0, min(NPG, P.d_ff - g * NPG));  // neurons owned
  const int r2 = P.d_model - P.r;
  // Synchronisation words that every gather workgroup would otherwise poll (the GS statistics
  // slots of a layer, the GG "written" words) sit in a few cache lines of one memory channel:
  // polled by all workgroups they turn that channel into a hot spot that throttles every
  // stream passing through it.  One leader per group of GG / 8 gather workgroups therefore
  // does the wide poll and republishes a single word for its group.
  constexpr int GPL = GG / kLeaders;  // gather workgroups per leader
  const int lead = g / GPL;
  const bool is_leader = g % GPL == lead % GPL;  // the leaders sit on different XCDs

  // ------------------------------------------------------------------------------ control
  if (wave < 2) {
    for (int l = wave; l < L; l += 2) {
      if (l >= kRing && !wait_ge(&sh.g.g_consumed[l % kRing], TW * (l / kRing), ab, W(1))) return;
      const uint32_t epoch = P.epoch_base + (uint32_t)l + 1u;
      const unsigned long long* sc = P.scores + (size_t)l * P.d_ff + (NPGg > 0 ? (size_t)g * NPG : 0);
      unsigned long long sv[MW];
      float theta;
      const long long tp = prof ? wall_clock64() : 0;
      {
        // the leader's theta and the workgroup's own scores, in one round trip
        const unsigned long long* tw = P.thetaw + ((size_t)l * kLeaders + lead) * kCell;
        SpinGuard guard;
        unsigned long long v;
        for (;;) {
          v = ld_u64(tw);
#pragma unroll
          for (int k = 0; k < MW; ++k) {
            const int n = lane + kWave * k;
            sv[k] = ld_u64(sc + (n < NPGg ? n : 0));
          }
          bool ok = hi32(v) == epoch;
#pragma unroll
          for (int k = 0; k < MW; ++k) ok = ok && (NPGg == 0 || hi32(sv[k]) == epoch);
          if (__all(ok)) break;
          if (guard.expired(ab, 2)) return;
          if (prof) pw[3] += 1;
          __builtin_amdgcn_s_sleep(2);
        }
        theta = lo_f32(uniform_u64(v));
      }
      if (prof) pw[2] += wall_clock64() - tp;
      unsigned long long mask[MW];
      int cnt = 0;
#pragma unroll
      for (int k = 0; k < MW; ++k) {
        const int n = lane + kWave * k;
        const float sval = lo_f32(sv[k]);
        mask[k] = __ballot(n < NPGg && sval > theta);
        cnt += __popcll(mask[k]);
        sh.g.a_ring[l % kRing][n] = sval - theta;
      }
      if (lane == 0) {
        st_u64(P.gcnt + (size_t)l * kMaxGather + g, ((unsigned long long)epoch << 32) | (uint32_t)cnt);
        sh.g.theta_ring[l % kRing] = theta;
#pragma unroll
        for (int k = 0; k < MW; ++k) {
          sh.g.mask_ring[l % kRing][k] = mask[k];
          sh.g.mask_hist[l][k] = mask[k];
        }
      }
      lds_fence();
      // layers are posted in order: wait for the other control wave to have posted l - 1
      if (!wait_ge(&sh.g.theta_ready, l, ab, W(5))) return;
      if (lane == 0) lds_signal_set(&sh.g.theta_ready, l + 1);
      mark(l);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ writer
  if (wave == 2) {
    const int DP = P.DP;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(P.part, (uint32_t)L * GG * DP * 4u);
    for (int l = 0; l < L; ++l) {
      f32x4 acc[FPL];
#pragma unroll
      for (int k = 0; k < FPL; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int o = l / kTeams;  // ordinal of the layer within its team
      for (int ti = 0; ti < TW; ++ti) {
        const int i = l % kTeams + kTeams * ti;
        const int slot = i * RB + o % RB;
        if (!wait_ge(&sh.g.row_full[slot], 2 * (o + 1), ab, W(1))) return;
        if (lds_read(&sh.g.row_full[slot]) & 1) {
          const float* row = rows + (size_t)slot * P.d_model;
#pragma unroll
          for (int k = 0; k < FPL; ++k) {
            const int f = lane + kWave * k;
            if (f * 4 < P.d_model) acc[k] += *reinterpret_cast<const f32x4*>(&row[f * 4]);
          }
        }
        lds_fence();
        if (lane == 0) lds_signal_set(&sh.g.row_free[i], o + 1);
      }
      const long long tc = prof ? wall_clock64() : 0;
      const uint32_t row_off = (uint32_t)(l * GG + g) * DP * 4u;
#pragma unroll
      for (int k = 0; k < FPL; ++k) {
        const int f = lane + kWave * k;
        if (f * 4 < DP) buf_store_f32x4(prs, row_off + (uint32_t)f * 16u, acc[k]);
      }
      wait_vmem();
      if (lane == 0) st_u64(P.gdone + g, ((unsigned long long)P.epoch_base << 32) | (uint32_t)(l + 1));
      if (prof) pw[2] += wall_clock64() - tc;
      mark(l);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ reduce
  if (wave < 5) {
    const int DP = P.DP, CWG = P.CWG;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(P.part, (uint32_t)L * GG * DP * 4u);
    const bool want_idx = P.idx || P.uidx || P.count || P.ucount;
    // The output columns are cut into slices of CWG floats (a whole number of 64-byte
    // sectors, so that a slice of a partial row is fetched without read amplification); the
    // first NR gather workgroups reduce one slice each.
    const bool reducer = g < P.NR;
    if (!reducer && !want_idx) {
      prof_flush();
      return;
    }
    for (int l = wave - 3; l < L; l += 2) {
      // every gather workgroup has written layer l: the leaders' group words say so.  The
      // two reduce waves share what they have seen, so a wave that is behind does not poll.
      if (reducer && lds_read(&sh.g.red_seen) < l + 1) {
        const long long tp = prof ? wall_clock64() : 0;
        SpinGuard guard;
        for (;;) {
          const unsigned long long v = ld_u64(P.gdone2 + (size_t)(lane < kLeaders ? lane : 0) * kCell);
          int m = hi32(v) == P.epoch_base ? (int)(uint32_t)v : 0;
#pragma unroll
          for (int o = 32; o >= 1; o >>= 1) m = min(m, __shfl_xor(m, o));
          if (m >= l + 1) {
            if (lane == 0) __hip_atomic_fetch_max((lds_int_t*)&sh.g.red_seen, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            break;
          }
          if (guard.expired(ab, 3)) return;
          __builtin_amdgcn_s_sleep(2);
        }
        if (prof) pw[1] += wall_clock64() - tp;
      }
      const long long tl = prof ? wall_clock64() : 0;
      unsigned long long cv[WPL];
#pragma unroll
      for (int j = 0; j < WPL; ++j) {
        const int wi = lane + kWave * j;
        cv[j] = want_idx ? ld_u64(P.gcnt + (size_t)l * kMaxGather + (wi < GG ? wi : 0)) : 0ull;
      }
      if (reducer) {
        f32x4 pv[WPL][CW4];
#pragma unroll
        for (int j = 0; j < WPL; ++j) {
          const int wi = lane + kWave * j;
          const uint32_t off = ((uint32_t)(l * GG + (wi < GG ? wi : 0)) * DP + (uint32_t)g * CWG) * 4u;
#pragma unroll
          for (int i = 0; i < CW4; ++i) pv[j][i] = buf_load_f32x4(prs, off + 16u * (i * 4 < CWG ? i : 0));
        }
#pragma unroll
        for (int i = 0; i < CW4; ++i) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float mine = 0.f;  // this lane's writers, in ascending workgroup order
#pragma unroll
            for (int j = 0; j < WPL; ++j) mine += (lane + kWave * j < GG) ? pv[j][i][e] : 0.f;
            const float tot = wave_sum_dpp(mine);
            const int col = g * CWG + i * 4 + e;
            if (lane == 0 && i * 4 + e < CWG && col < P.d_model) P.y[(size_t)l * P.d_model + col] = tot;
          }
        }
      }
      if (prof) pw[2] += wall_clock64() - tl;
      mark(l);
      if (!want_idx) continue;
      // compacted ascending index list: counts of all gather workgroups were published long ago
      {
        SpinGuard guard;
        const uint32_t epoch = P.epoch_base + (uint32_t)l + 1u;
        for (;;) {
          bool ok = true;
#pragma unroll
          for (int j = 0; j < WPL; ++j) ok = ok && hi32(cv[j]) == epoch;
          if (__all(ok)) break;
          if (guard.expired(ab, 4)) return;
#pragma unroll
          for (int j = 0; j < WPL; ++j) {
            const int wi = lane + kWave * j;
            cv[j] = ld_u64(P.gcnt + (size_t)l * kMaxGather + (wi < GG ? wi : 0));
          }
        }
      }
      int before = 0, all = 0;
#pragma unroll
      for (int j = 0; j < WPL; ++j) {
        const int wi = lane + kWave * j;
        const int cn = wi < GG ? (int)(uint32_t)cv[j] : 0;
        before += wi < g ? cn : 0;
        all += cn;
      }
      const int off_g = wave_sum_int(before);
      const int total = wave_sum_int(all);
      int below = off_g;
#pragma unroll
      for (int k = 0; k < MW; ++k) {
        const unsigned long long mk = sh.g.mask_hist[l][k];
        if ((mk >> lane) & 1ull) {
          const int pos = below + lanes_below(mk);
          const int j = g * NPG + lane + kWave * k;
          if (P.idx) P.idx[(size_t)l * P.d_ff + pos] = j;
          if (P.uidx) P.uidx[(size_t)l * P.d_ff + pos] = j;
        }
        below += __popcll(mk);
      }
      if (g == 0 && lane == 0) {
        if (P.count) P.count[l] = total;
        if (P.ucount) P.ucount[l] = total;
      }
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ gather
  // The active neurons of a layer are dealt to the gather waves round-robin (rotated from
  // layer to layer so that every wave gets its share of idle layers).  A wave handles its
  // neurons one at a time and adds them into its LDS row of the layer; RB rows per wave let
  // it run ahead of the writer by RB - 1 layers.
  if (wave < 5 + NGW) {
    const int gw = wave - 5;
    const int nvec2 = r2 / VEC, nvecv = P.d_model / VEC;
    uint32_t koff[CPL2], voff[CPLV];  // byte offsets of this lane's chunks inside a row
#pragma unroll
    for (int c = 0; c < CPL2; ++c) {
      const int ch = lane + kWave * c;
      koff[c] = (uint32_t)(ch < nvec2 ? ch : 0) * VEC * (uint32_t)sizeof(WT);
      if (gw == 0) {  // one wave fills the shared copy of q[r:]
        float qv[VEC];
        load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)P.r + (int64_t)(ch < nvec2 ? ch : 0) * VEC, qv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) q2s[ch * VEC + e] = ch < nvec2 ? qv[e] : 0.f;
      }
    }
#pragma unroll
    for (int c = 0; c < CPLV; ++c) {
      const int ch = lane + kWave * c;
      voff[c] = (uint32_t)(ch < nvecv ? ch : 0) * VEC * (uint32_t)sizeof(WT);
    }
    if (gw == 0) {
      lds_fence();
      if (lane == 0) lds_signal_set(&sh.g.q2_ready, 1);
    }
    if (!wait_ge(&sh.g.q2_ready, 1, ab)) return;
    const uint32_t k2_bytes = (uint32_t)P.d_ff * (uint32_t)r2 * (uint32_t)sizeof(WT);
    const uint32_t v_bytes = (uint32_t)P.d_ff * (uint32_t)P.d_model * (uint32_t)sizeof(WT);

    const int team = gw % kTeams, gt = gw / kTeams;  // team, and index within the team
    for (int l = team; l < L; l += kTeams) {
      if (!wait_ge(&sh.g.theta_ready, l + 1, ab, W(1))) return;
      const int o = l / kTeams;  // ordinal of the layer within the team
      const int slot = gw * RB + o % RB;
      float* myrow = rows + (size_t)slot * P.d_model;
      // This wave's neurons of the layer: every TW-th active one, starting at a position
      // that rotates with the layer.  They are handled two at a time (both row pairs are
      // requested before either is used), so that a layer with up to 2 * TW active neurons
      // costs the workgroup one memory round trip.
      int first = gt - (o * 3) % TW;  // position of the wave's first neuron among the active ones
      if (first < 0) first += TW;
      unsigned long long mk[MW];
#pragma unroll
      for (int k = 0; k < MW; ++k) mk[k] = uniform_u64(sh.g.mask_ring[l % kRing][k]);
      int skip = first, mine = 0;
      // Pops the wave's next neuron (local index) from the masks, -1 when there is none.
      auto next_neuron = [&]() -> int {
#pragma unroll
        for (int k = 0; k < MW; ++k) {
          while (mk[k]) {
            const int nl = __builtin_ctzll(mk[k]);
            mk[k] &= mk[k] - 1;
            if (skip == 0) {
              skip = TW - 1;
              return kWave * k + nl;
            }
            --skip;
          }
        }
        return -1;
      };
      for (;;) {
        const int n0 = next_neuron();
        if (n0 < 0) break;
        const int n1 = next_neuron();
        const long long tq0 = prof ? wall_clock64() : 0;
        // a missing second neuron reads through a descriptor without records: zeros, no traffic
        const __amdgpu_buffer_rsrc_t kb0 = make_rsrc(P.k2n[l], k2_bytes), vb0 = make_rsrc(P.vn[l], v_bytes);
        const __amdgpu_buffer_rsrc_t kb1 = make_rsrc(P.k2n[l], n1 >= 0 ? k2_bytes : 0u);
        const __amdgpu_buffer_rsrc_t vb1 = make_rsrc(P.vn[l], n1 >= 0 ? v_bytes : 0u);
        const uint32_t j0 = (uint32_t)(g * NPG + n0), j1 = (uint32_t)(g * NPG + (n1 >= 0 ? n1 : n0));
        Vec16<WT> kr0[CPL2], vr0[CPLV], kr1[CPL2], vr1[CPLV];
#pragma unroll
        for (int c = 0; c < CPL2; ++c) kr0[c] = buf_load_w<WT>(kb0, koff[c], j0 * (uint32_t)r2 * (uint32_t)sizeof(WT));
#pragma unroll
        for (int c = 0; c < CPL2; ++c) kr1[c] = buf_load_w<WT>(kb1, koff[c], j1 * (uint32_t)r2 * (uint32_t)sizeof(WT));
#pragma unroll
        for (int c = 0; c < CPLV; ++c) vr0[c] = buf_load_w<WT>(vb0, voff[c], j0 * (uint32_t)P.d_model * (uint32_t)sizeof(WT));
#pragma unroll
        for (int c = 0; c < CPLV; ++c) vr1[c] = buf_load_w<WT>(vb1, voff[c], j1 * (uint32_t)P.d_model * (uint32_t)sizeof(WT));
        float gd0 = 0.f, gd1 = 0.f;
#pragma unroll
        for (int c = 0; c < CPL2; ++c) {
          const float* qp = &q2s[(lane + kWave * c) * VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            gd0 += kr0[c].get(e) * qp[e];
            gd1 += kr1[c].get(e) * qp[e];
          }
        }
        gd0 = wave_sum_dpp(gd0);
        gd1 = wave_sum_dpp(gd1);
        const float u0 = gelu(sh.g.a_ring[l % kRing][n0], P.gelu) * gd0;
        const float u1 = n1 >= 0 ? gelu(sh.g.a_ring[l % kRing][n1], P.gelu) * gd1 : 0.f;
        if (prof) pw[3] += wall_clock64() - tq0;
        // the wave's LDS row of this layer: the first neuron overwrites it (once the writer
        // has drained the layer that used the row before), later ones add to it
        if (mine == 0 && o >= RB && !wait_ge(&sh.g.row_free[gw], o - RB + 1, ab, W(2))) return;
#pragma unroll
        for (int c = 0; c < CPLV; ++c) {
          const int ch = lane + kWave * c;
          float* dst = myrow + (size_t)ch * VEC;
          if (ch < nvecv) {
#pragma unroll
            for (int e = 0; e < VEC; e += 4) {
              // neurons are added in ascending order, one after the other (u1 = 0 adds +0)
              f32x4 t{u0 * vr0[c].get(e), u0 * vr0[c].get(e + 1), u0 * vr0[c].get(e + 2), u0 * vr0[c].get(e + 3)};
              if (mine) t += *reinterpret_cast<const f32x4*>(dst + e);
              if (n1 >= 0) t += f32x4{u1 * vr1[c].get(e), u1 * vr1[c].get(e + 1), u1 * vr1[c].get(e + 2), u1 * vr1[c].get(e + 3)};
              *reinterpret_cast<f32x4*>(dst + e) = t;
            }
          }
        }
        mine += 2;
        if (prof) pw[5] += wall_clock64() - tq0;
      }
      lds_fence();
      if (lane == 0) lds_signal_add(&sh.g.g_consumed[l % kRing]);
      // the slot's previous posting must have been read before it is overwritten
      if (mine == 0 && o >= RB && !wait_ge(&sh.g.row_free[gw], o - RB + 1, ab, W(2))) return;
      if (lane == 0) lds_signal_set(&sh.g.row_full[slot], 2 * (o + 1) + (mine ? 1 : 0));
      mark(l);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ leader
  // In a leader workgroup: merges the stream workgroups' statistics of every layer into
  // theta and publishes it for the group, as fast as the stream delivers (it depends on
  // nothing downstream, so a workgroup that is behind never holds up its group's theta).
  if (wave == 6 + NGW && is_leader) {
    for (int l = 0; l < L; ++l) {
      const uint32_t epoch = P.epoch_base + (uint32_t)l + 1u;
      const unsigned long long* st = P.stats + (size_t)l * kStatSlots * 2;
      unsigned long long m0[SPL], m1[SPL];
      SpinGuard guard;
      for (;;) {
#pragma unroll
        for (int k = 0; k < SPL; ++k) {
          const int t = lane + kWave * k;
          const unsigned long long* sp = st + (size_t)(t < GS ? t : 0) * 2;
          m0[k] = ld_u64(sp);
          m1[k] = ld_u64(sp + 1);
        }
        bool ok = true;
#pragma unroll
        for (int k = 0; k < SPL; ++k) ok = ok && hi32(m0[k]) == epoch && hi32(m1[k]) == epoch;
        if (__all(ok)) break;
        if (guard.expired(ab, 2)) return;
        if (prof) pw[3] += 1;
      }
      // merge (Chan et al.): mean = sum n_s mean_s / n, M2 = sum M2_s + n_s (mean_s - mean)^2
      float s1 = 0.f;
#pragma unroll
      for (int k = 0; k < SPL; ++k) {
        const int t = lane + kWave * k;
        const int ns = t < GS ? max(0, min(P.RS, P.d_ff - t * P.RS)) : 0;
        s1 += (float)ns * lo_f32(m0[k]);
      }
      const float mean = wave_sum_dpp(s1) / (float)P.d_ff;
      float m2 = 0.f;
#pragma unroll
      for (int k = 0; k < SPL; ++k) {
        const int t = lane + kWave * k;
        const int ns = t < GS ? max(0, min(P.RS, P.d_ff - t * P.RS)) : 0;
        const float d = lo_f32(m0[k]) - mean;
        m2 += (t < GS ? lo_f32(m1[k]) : 0.f) + (float)ns * d * d;
      }
      m2 = wave_sum_dpp(m2);
      const float theta = mean + sqrtf(m2 / (float)(P.d_ff - 1)) * P.z;
      if (lane == 0) {
        st_u64(P.thetaw + ((size_t)l * kLeaders + lead) * kCell, pack(theta, epoch));
        if (lead == 0 && P.theta) P.theta[l] = theta;
      }
      mark(l);
    }
    prof_flush();
    return;
  }

  // ------------------------------------------------------------------------------ collector
  // In a leader workgroup: republishes min(layers written) over the group's writers.
  if (wave == 5 + NGW && is_leader) {
    int published = 0;
    SpinGuard guard;
    while (published < L) {
      const unsigned long long v = ld_u64(P.gdone + lead * GPL + (lane < GPL ? lane : 0));
      const int done = hi32(v) == P.epoch_base ? (int)(uint32_t)v : 0;
      int m = done;
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) m = min(m, __shfl_xor(m, o));
      if (m > published) {
        published = m;
        if (lane == 0) st_u64(P.gdone2 + (size_t)lead * kCell, ((unsigned long long)P.epoch_base << 32) | (uint32_t)m);
        guard = SpinGuard();
      } else {
        if (guard.expired(ab, 6)) return;
        __builtin_amdgcn_s_sleep(2);
      }
    }
    prof_flush();
  }
}

template <typename WT, bool QB, int GP, int CPL1, int CPL2, int CPLV, int RPW, int RIF, int NS, int NGW, int RB, int CW4>
hipError_t launch_variant(const SpecParams& P, hipStream_t st) {
  const void* kern = P.prof ? reinterpret_cast<const void*>(ffn_spec_kernel<WT, QB, GP, CPL1, CPL2, CPLV, RPW, RIF, NS, NGW, RB, CW4, true>)
                            : reinterpret_cast<const void*>(ffn_spec_kernel<WT, QB, GP, CPL1, CPL2, CPLV, RPW, RIF, NS, NGW, RB, CW4, false>);
  const size_t dyn = (size_t)NGW * RB * (size_t)P.d_model * sizeof(float);
  hipError_t err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
  if (err != hipSuccess) return err;
  void* args[] = {const_cast<SpecParams*>(&P)};
  constexpr int waves = (NS + 1 > NGW + 7) ? NS + 1 : NGW + 7;
  // A plain launch: every workgroup needs a compute unit of its own (the LDS request makes
  // sure of that) and all of them must be resident together, which holds when the device has
  // kG compute units and no other kernel is running on it.  If it does not hold, the
  // bounded waits give up and the status word reports it.  (A cooperative launch would only
  // add the occupancy check that fused_supported() already makes, at several times the
  // launch latency.)
  return hipLaunchKernel(kern, dim3(kG), dim3(waves * kWave), args, dyn, st);
}

uint32_t next_epoch_base(int n_layers) {
  // Process-wide counter: every launch gets epochs no earlier launch has written into a
  // workspace, so stale words can never be mistaken for fresh ones.
  static std::atomic<uint32_t> counter{1u};
  uint32_t b = counter.fetch_add((uint32_t)n_layers + 64u);
  if (b == 0) b = counter.fetch_add((uint32_t)n_layers + 64u);  // the tag 0 is never used
  return b;
}

int g_fused_profile = 0;

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct ScratchLayout {
  size_t status, stats, scores, gcnt, gdone, thetaw, gdone2, part, prof, total;
};

// Sized for the variant with the most gather workgroups (a partial row is at most
// d_model + 4 * kMaxGather floats long), so the size depends on the shape only.
ScratchLayout scratch_layout(int d_model, int d_ff) {
  ScratchLayout s;
  size_t o = 0;
  s.status = o; o += 256;
  s.stats = o;  o += align256((size_t)kFusedMaxLayers * kStatSlots * 2 * 8);
  s.scores = o; o += align256((size_t)kFusedMaxLayers * (size_t)d_ff * 8);
  s.gcnt = o;   o += align256((size_t)kFusedMaxLayers * kMaxGather * 8);
  s.gdone = o;  o += align256((size_t)kMaxGather * 8);
  s.thetaw = o; o += align256((size_t)kFusedMaxLayers * kLeaders * kCell * 8);
  s.gdone2 = o; o += align256((size_t)kLeaders * kCell * 8);
  s.part = o;   o += align256((size_t)kFusedMaxLayers * kMaxGather * ((size_t)d_model + 4 * kMaxGather) * 4);
  s.prof = o;   o += kProfBytes;
  s.total = o;
  return s;
}

// The compiled variants and their shape limits.
struct Variant {
  int bf16, gp, cpl1, cpl2, cplv, rpw, rif, ns, ngw, rb, cw4;
};
constexpr Variant kVariants[] = {
    {1, 16, 2, 3, 5, 6, 3, 12, 8, 2, 8},    // Gemma-2 2B class
    {1, 16, 2, 3, 5, 8, 4, 14, 8, 2, 8},    // the same with the wider d_ff of the paper's 2B model
    {1, 16, 3, 4, 7, 8, 3, 14, 8, 1, 8},    // Gemma-2 9B class
    {0, 8, 4, 5, 9, 4, 2, 12, 8, 1, 12},    // fp32 weights
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr size_t kMaxRowBytes = 148 * 1024;  // dynamic LDS left for the gather waves' rows

struct Split {
  int GS, GG, RS, NPG, CWG, NR, DP;
};
Split split_for(const Variant& v, int d_model, int d_ff) {
  Split s;
  s.GS = kG / kGroup * (kGroup - v.gp);
  s.GG = kG / kGroup * v.gp;
  s.RS = (d_ff + s.GS - 1) / s.GS;
  s.NPG = (d_ff + s.GG - 1) / s.GG;
  s.CWG = ((d_model + s.GG - 1) / s.GG + 15) / 16 * 16;
  s.NR = (d_model + s.CWG - 1) / s.CWG;
  s.DP = s.CWG * s.NR;
  return s;
}

// Returns -1 when no variant fits.
int spec_variant(const FfnProblem& p) {
  const int vec = p.w_bf16 ? 8 : 4;
  const int c1 = (p.r / vec + kWave - 1) / kWave, c2 = ((p.d_model - p.r) / vec + kWave - 1) / kWave;
  const int cv = (p.d_model / vec + kWave - 1) / kWave;
  for (int i = 0; i < kNumVariants; ++i) {
    const Variant& v = kVariants[i];
    if (v.bf16 != (p.w_bf16 ? 1 : 0)) continue;
    const Split s = split_for(v, p.d_model, p.d_ff);
    if (c1 > v.cpl1 || c2 > v.cpl2 || cv > v.cplv) continue;
    if (s.RS > v.rpw * v.ns || s.NPG > mask_words(v.gp) * kWave) continue;
    if (s.CWG > v.cw4 * 4 || s.DP > v.cplv * vec * kWave) continue;
    if ((size_t)v.ngw * v.rb * p.d_model * sizeof(float) > kMaxRowBytes) continue;
    return i;
  }
  return -1;
}

template <int I>
hipError_t launch_index(const SpecParams& P, hipStream_t st) {
  constexpr Variant v = kVariants[I];
  if constexpr (v.bf16) {
    if (P.q_bf16) return launch_variant<bf16_t, true, v.gp, v.cpl1, v.cpl2, v.cplv, v.rpw, v.rif, v.ns, v.ngw, v.rb, v.cw4>(P, st);
    return launch_variant<bf16_t, false, v.gp, v.cpl1, v.cpl2, v.cplv, v.rpw, v.rif, v.ns, v.ngw, v.rb, v.cw4>(P, st);
  } else {
    return launch_variant<float, false, v.gp, v.cpl1, v.cpl2, v.cplv, v.rpw, v.rif, v.ns, v.ngw, v.rb, v.cw4>(P, st);
  }
}

}  // namespace

void fused_set_profile(int on) { g_fused_profile = on; }
size_t fused_profile_offset(int d_model, int d_ff) { return scratch_layout(d_model, d_ff).prof; }
size_t fused_profile_bytes() { return kProfBytes; }
size_t fused_scratch_bytes(int d_model, int d_ff) { return scratch_layout(d_model, d_ff).total; }

// One workgroup per compute unit: the current device must have at least kG of them.
static bool device_has_room() {
  static std::atomic<int> cached[64];  // per device: 0 unknown, 1 yes, 2 no
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  int c = cached[dev].load();
  if (c == 0) {
    int cus = 0;
    const bool ok = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= kG;
    c = ok ? 1 : 2;
    cached[dev].store(c);
  }
  return c == 1;
}

bool fused_supported(const FfnProblem& p, int n_layers) {
  return p.batch == 1 && n_layers >= 1 && spec_variant(p) >= 0 && device_has_room();
}

// layers: n_layers problems that differ only in weights and outputs' leading index.
hipError_t launch_ffn_fused(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                            const void* const* vn, int n_layers, void* scratch, hipStream_t st) {
  hipError_t err = hipSuccess;
  const ScratchLayout lay = scratch_layout(p0.d_model, p0.d_ff);
  const int vi = spec_variant(p0);
  if (vi < 0) return hipErrorInvalidValue;
  const Split sp = split_for(kVariants[vi], p0.d_model, p0.d_ff);
  char* s = static_cast<char*>(scratch);
  for (int base = 0; base < n_layers && err == hipSuccess; base += kFusedMaxLayers) {
    const int L = min(kFusedMaxLayers, n_layers - base);
    SpecParams P;
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
    P.status = reinterpret_cast<int32_t*>(s + lay.status);
    P.stats = reinterpret_cast<unsigned long long*>(s + lay.stats);
    P.scores = reinterpret_cast<unsigned long long*>(s + lay.scores);
    P.gcnt = reinterpret_cast<unsigned long long*>(s + lay.gcnt);
    P.gdone = reinterpret_cast<unsigned long long*>(s + lay.gdone);
    P.thetaw = reinterpret_cast<unsigned long long*>(s + lay.thetaw);
    P.gdone2 = reinterpret_cast<unsigned long long*>(s + lay.gdone2);
    P.part = reinterpret_cast<float*>(s + lay.part);
    P.prof = g_fused_profile ? reinterpret_cast<long long*>(s + lay.prof) : nullptr;
    P.n_layers = L;
    P.d_model = p0.d_model;
    P.d_ff = p0.d_ff;
    P.r = p0.r;
    P.q_bf16 = p0.q_bf16;
    P.gelu = p0.gelu;
    P.z = p0.z;
    P.RS = sp.RS;
    P.NPG = sp.NPG;
    P.CWG = sp.CWG;
    P.NR = sp.NR;
    P.DP = sp.DP;
    P.epoch_base = next_epoch_base(L);
    switch (vi) {
      case 0: err = launch_index<0>(P, st); break;
      case 1: err = launch_index<1>(P, st); break;
      case 2: err = launch_index<2>(P, st); break;
      case 3: err = launch_index<3>(P, st); break;
      default: err = hipErrorInvalidValue; break;
    }
  }
  return err;
}

}  // namespace spark
