// Spark-FFN decode (Eq.2 of arXiv 2506.06644) for one token and a stack of independent
// layers, phase by phase over the whole stack (gfx950).
//
// The layers of one call all read the same token and do not feed each other, so every step
// of the method can run for all layers at once, each as an ordinary bandwidth-bound launch:
//
//   predict   s[l][j] = K1n_l[j] . q[:r] for every neuron of every layer: one sweep over all
//             the K1n (the 2 r d_ff term of Eq.4, four fifths of the bytes).  A workgroup
//             also leaves the (mean, M2) of its own scores.
//   gather    one workgroup per (layer, block of neurons): merges the layer's statistics in a
//             fixed order into theta = mean + std * Q(1 - k/d_ff) (Eq.11), finds the block's
//             active neurons (s > theta, strict), and for those only reads the K2n row and
//             the Vn row (one contiguous burst each): g = K2n[j] . q[r:],
//             u = GELU(s_j - theta) * g, acc += u * Vn[j][:].  The block's partial output
//             row goes to the workspace.
//   reduce    y[l][:] = sum of the layer's partial rows in block order.
//   select    (only when the caller wants them) theta, count and the ascending index list.
//
// Nothing waits on anything inside a launch: no co-residency requirement, no spinning.  All
// sums have a fixed order, so results are reproducible bit for bit, and every workgroup of
// a layer derives theta from the same numbers in the same order, hence identically.
#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kMaxRPB = 256;  // most predictor rows per workgroup
constexpr int kMaxNBC = 64;   // gather blocks per layer the scratch is sized for at the full layer count
constexpr int kMostNBC = 128;  // most gather blocks per layer (short stacks use the spare partial rows)

struct PhasedParams {
  const void* k1n[kPhasedMaxLayers];
  const void* k2n[kPhasedMaxLayers];
  const void* vn[kPhasedMaxLayers];
  const void* q;
  float* y;            // [L][d_model]
  float* theta;        // [L]        optional
  int32_t* count;      // [L]        optional
  int32_t* idx;        // [L][d_ff]  optional
  int32_t* ucount;     // [L]        optional
  int32_t* uidx;       // [L][d_ff]  optional
  float* scores;       // [L][d_ff]
  float* stats;        // [L][NBA][2]  (mean, M2) of each predictor block
  float* part;         // [L][NBC][d_model]
  int n_layers, d_model, d_ff, r, q_bf16, gelu;
  int dense;  // every neuron's K2n and Vn row is read (inactive ones contribute an exact zero)
  float z;
  int RPB;  // predictor rows per workgroup (multiple of 16, <= kMaxRPB)
  int NBA;  // predictor workgroups per layer, ceil(d_ff / RPB)
  int NPB;  // neurons per gather workgroup (multiple of 64)
  int NBC;  // gather workgroups per layer, ceil(d_ff / NPB)
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
// a.lo * b.lo + a.hi * b.hi + c on packed bf16 pairs (bf16 products are exact in fp32)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// Sum over the wavefront with DPP moves (quad swaps, row mirrors, row broadcasts); the total
// is returned as a uniform value.  The order of additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return x + __int_as_float(t);
}
__device__ __forceinline__ float wave_total(float x) {
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

template <typename WT>
__device__ __forceinline__ Vec16<WT> load_stream(const WT* p) {
  Vec16<WT> v;
  v.raw = __builtin_nontemporal_load(reinterpret_cast<const decltype(v.raw)*>(p));
  return v;
}

// Per-row scale of an 8-bit weight array: the fp32 scales follow the last row of codes.  Other
// weight types carry no scale.
template <typename WT>
__device__ __forceinline__ const float* row_scales(const void* w, int rows, int cols) {
  if constexpr (sizeof(WT) == 1) return reinterpret_cast<const float*>(static_cast<const char*>(w) + (size_t)rows * (size_t)cols);
  else return nullptr;
}

// Rows of one predictor block that are real neurons (the last block of a layer may be short).
__device__ __forceinline__ int rows_in_block(int blk, int rpb, int d_ff) { return max(0, min(rpb, d_ff - blk * rpb)); }

// theta of layer l from the predictor blocks' (mean, M2): the pairwise update of Chan et al.
// with every block against the global mean, mean = sum n_b mean_b / n,
// M2 = sum (M2_b + n_b (mean_b - mean)^2), evaluated by one wavefront in a fixed order.
__device__ __forceinline__ float layer_theta(const PhasedParams& P, int l, int lane) {
  const float* st = P.stats + (size_t)l * P.NBA * 2;
  float s1 = 0.f;
  for (int b = lane; b < P.NBA; b += kWave) s1 += (float)rows_in_block(b, P.RPB, P.d_ff) * st[2 * b];
  const float mean = wave_total(s1) / (float)P.d_ff;
  float m2 = 0.f;
  for (int b = lane; b < P.NBA; b += kWave) {
    const float d = st[2 * b] - mean;
    m2 += st[2 * b + 1] + (float)rows_in_block(b, P.RPB, P.d_ff) * d * d;
  }
  m2 = wave_total(m2);
  return mean + sqrtf(m2 / (float)(P.d_ff - 1)) * P.z;
}

// --------------------------------------------------------------------------------- predict
// Workgroup (4 waves) = RPB consecutive neurons of one layer, swept 16 rows at a time: each
// wave reads four consecutive rows of the 16 (4 * CPL1 16-byte loads in flight per lane;
// occupancy does the rest of the latency hiding), so the workgroup as a whole walks through
// one contiguous stretch of memory.
// R = rows a wave has in flight: 4 when many workgroups share a compute unit, 12 (a block of
// 48 rows in a single sweep) when a call has so few layers that a workgroup is alone on its
// compute unit and its own loads are all the latency hiding there is.
template <typename WT, bool QB, int CPL1, int R = 4>
__global__ __launch_bounds__(256) void predict_layers_kernel(const PhasedParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr bool DOT2 = QB && VEC == 8;
  __shared__ float s_sh[kMaxRPB];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int l = blockIdx.y, blk = blockIdx.x;
  const int nvec1 = P.r / VEC;
  const int row0 = blk * P.RPB, nrows = rows_in_block(blk, P.RPB, P.d_ff);
  const int rpw = P.RPB / 4;

  float q1[DOT2 ? 1 : CPL1][VEC];
  u32x4 q1p[DOT2 ? CPL1 : 1];
#pragma unroll
  for (int c = 0; c < CPL1; ++c) {
    const int ch = lane + kWave * c;
    const int co = (ch < nvec1 ? ch : 0) * VEC;
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
  }

  const WT* base = static_cast<const WT*>(P.k1n[l]);
  const float* scales = row_scales<WT>(P.k1n[l], P.d_ff, P.r);
  for (int i = 0; i < rpw; i += R) {
    Vec16<WT> reg[R][CPL1];
    float sc[R];
#pragma unroll
    for (int e = 0; e < R; ++e) {
      const int lr = i * 4 + wave * R + e;
      // rows past the end of the layer re-read the block's first row; the value is dropped
      const WT* row = base + (size_t)(row0 + (lr < nrows ? lr : 0)) * P.r;
      sc[e] = 1.f;
      if constexpr (sizeof(WT) == 1) sc[e] = scales[row0 + (lr < nrows ? lr : 0)];
#pragma unroll
      for (int c = 0; c < CPL1; ++c) {
        const int ch = lane + kWave * c;
        reg[e][c] = load_stream<WT>(row + (size_t)(ch < nvec1 ? ch : 0) * VEC);
      }
    }
#pragma unroll
    for (int e = 0; e < R; ++e) {
      float acc = 0.f;
      if constexpr (DOT2) {
        float accc[CPL1];
#pragma unroll
        for (int c = 0; c < CPL1; ++c) {
          accc[c] = 0.f;
#pragma unroll
          for (int d = 0; d < 4; ++d) accc[c] = dot2_bf16(reg[e][c].raw[d], q1p[c][d], accc[c]);
        }
#pragma unroll
        for (int c = 0; c < CPL1; ++c) acc += accc[c];
      } else {
#pragma unroll
        for (int c = 0; c < CPL1; ++c)
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc += reg[e][c].get(v) * q1[c][v];
      }
      acc = wave_total(acc);
      const int lr = i * 4 + wave * R + e;
      if (lane == 0 && lr < nrows) s_sh[lr] = acc * sc[e];
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < nrows; t += 256) P.scores[(size_t)l * P.d_ff + row0 + t] = s_sh[t];
  if (wave == 0) {
    float v[kMaxRPB / kWave];
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < kMaxRPB / kWave; ++k) {
      const int t = lane + kWave * k;
      v[k] = t < nrows ? s_sh[t] : 0.f;
      sum += v[k];
    }
    float mean_b = 0.f, m2_b = 0.f;
    if (nrows > 0) {
      mean_b = wave_total(sum) / (float)nrows;
      float sq = 0.f;
#pragma unroll
      for (int k = 0; k < kMaxRPB / kWave; ++k) {
        const float d = lane + kWave * k < nrows ? v[k] - mean_b : 0.f;
        sq += d * d;
      }
      m2_b = wave_total(sq);
    }
    if (lane == 0) {
      float* st = P.stats + ((size_t)l * P.NBA + blk) * 2;
      st[0] = mean_b;
      st[1] = m2_b;
    }
  }
}

// ---------------------------------------------------------------------------------- gather
// 16-byte load of chunk `ch` of a weight row through a buffer descriptor that spans exactly
// that row (or nothing): chunks past the end of the row, and every chunk of a row that does
// not exist, come back as zeros without touching memory, so the loads need no branches and
// their number in flight is a compile-time constant.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_rsrc(const void* row, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(row), 0, (int)bytes, 0x00020000);
}
template <typename WT>
__device__ __forceinline__ Vec16<WT> row_load(__amdgpu_buffer_rsrc_t r, int ch) {
  Vec16<WT> v;
  const u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(r, ch * 16, 0, 0);
  v.raw = __builtin_bit_cast(decltype(v.raw), u);
  return v;
}

// Workgroup (NW waves) = NPB consecutive neurons of one layer.  The active neurons of the
// block are dealt to the waves round-robin in ascending order.  A wave always has the rows of
// its next neuron in flight while it works on the current one (two register buffers) and
// accumulates into registers; the waves' rows are then summed through LDS as a binary tree
// in a fixed order.
template <typename WT, int CPL2, int CPLV, int NW, int OCC>
__global__ __launch_bounds__(NW * kWave, OCC) void gather_layers_kernel(const PhasedParams P) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int MAXW = 16;  // mask words: NPB <= 1024
  constexpr int SPW = (MAXW + NW - 1) / NW;
  static_assert((NW & (NW - 1)) == 0 && NW >= 2, "tree reduction");
  __shared__ unsigned long long maskw[MAXW];
  __shared__ float s_blk[MAXW * kWave];
  extern __shared__ __align__(16) float dyn[];  // q[r:] as fp32 (CPL2 * 64 * VEC), then NW/2 rows of d_model
  float* q2s = dyn;
  float* rows = dyn + CPL2 * kWave * VEC;

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int l = blockIdx.y, blk = blockIdx.x;
  const int r2 = P.d_model - P.r;
  const int nvec2 = r2 / VEC, nvecv = P.d_model / VEC;
  const int n0 = blk * P.NPB, nn = max(0, min(P.NPB, P.d_ff - n0));
  const int nwords = P.NPB / kWave;

  // scores of the block (requested before the statistics are needed)
  float sv[SPW];
#pragma unroll
  for (int k = 0; k < SPW; ++k) {
    const int wd = wave + NW * k;  // mask word handled by this wave
    const int n = wd * kWave + lane;
    sv[k] = (wd < nwords && n < nn) ? P.scores[(size_t)l * P.d_ff + n0 + n] : 0.f;
  }
  for (int c = tid; c < CPL2 * kWave; c += NW * kWave) {
    float qv[VEC];
    load_q_vec<VEC>(P.q, P.q_bf16, (int64_t)P.r + (int64_t)(c < nvec2 ? c : 0) * VEC, qv);
#pragma unroll
    for (int e = 0; e < VEC; ++e) q2s[c * VEC + e] = c < nvec2 ? qv[e] : 0.f;
  }
  const float theta = layer_theta(P, l, lane);
#pragma unroll
  for (int k = 0; k < SPW; ++k) {
    const int wd = wave + NW * k;
    if (wd < nwords) {
      const int n = wd * kWave + lane;
      const unsigned long long m = __ballot(n < nn && (P.dense || sv[k] > theta));
      s_blk[n] = sv[k] - theta;
      if (lane == 0) maskw[wd] = m;
    }
  }
  if (blk == 0 && tid == 0 && P.theta) P.theta[l] = theta;
  __syncthreads();

  float acc[CPLV][VEC];
#pragma unroll
  for (int c = 0; c < CPLV; ++c)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[c][e] = 0.f;

  const WT* k2 = static_cast<const WT*>(P.k2n[l]);
  const WT* vn = static_cast<const WT*>(P.vn[l]);
  constexpr bool SCALED = sizeof(WT) == 1;
  const float* k2_scales = row_scales<WT>(P.k2n[l], P.d_ff, r2);
  const float* vn_scales = row_scales<WT>(P.vn[l], P.d_ff, P.d_model);
  // pops this wave's next active neuron (index inside the block), -1 when there is none
  int wd = 0, skip = wave;
  unsigned long long cur = nwords > 0 ? uniform_u64(maskw[0]) : 0ull;
  auto next_neuron = [&]() -> int {
    for (;;) {
      while (cur) {
        const int b = __builtin_ctzll(cur);
        cur &= cur - 1;
        if (skip == 0) {
          skip = NW - 1;
          return wd * kWave + b;
        }
        --skip;
      }
      if (++wd >= nwords) return -1;
      cur = uniform_u64(maskw[wd]);
    }
  };
  // (8-bit weights: the row's two scales travel with it, as the product scale_k2 * scale_v, which
  // is all the sum needs: u_j * Vn[j] = GELU(a) * (scale_k2 g) * (scale_v codes))
  auto request = [&](int n, Vec16<WT>(&kr)[CPL2], Vec16<WT>(&vr)[CPLV], float& sc) {
    const size_t j = (size_t)(n0 + (n >= 0 ? n : 0));
    const __amdgpu_buffer_rsrc_t kb = row_rsrc(k2 + j * r2, n >= 0 ? (uint32_t)r2 * (uint32_t)sizeof(WT) : 0u);
    const __amdgpu_buffer_rsrc_t vb = row_rsrc(vn + j * P.d_model, n >= 0 ? (uint32_t)P.d_model * (uint32_t)sizeof(WT) : 0u);
#pragma unroll
    for (int c = 0; c < CPL2; ++c) kr[c] = row_load<WT>(kb, lane + kWave * c);
#pragma unroll
    for (int c = 0; c < CPLV; ++c) vr[c] = row_load<WT>(vb, lane + kWave * c);
    sc = 1.f;
    if constexpr (SCALED) sc = k2_scales[j] * vn_scales[j];
  };
  auto consume = [&](int n, const Vec16<WT>(&kr)[CPL2], const Vec16<WT>(&vr)[CPLV], float sc) {
    float gd = 0.f;
#pragma unroll
    for (int c = 0; c < CPL2; ++c) {
      const float* qp = &q2s[(lane + kWave * c) * VEC];  // zero past the end of q[r:]
#pragma unroll
      for (int e = 0; e < VEC; ++e) gd += kr[c].get(e) * qp[e];
    }
    gd = wave_total(gd);
    const float a = n >= 0 ? s_blk[n] : 0.f;  // s_j - theta
    const float u = a > 0.f ? gelu(a, P.gelu) * (gd * sc) : 0.f;
#pragma unroll
    for (int c = 0; c < CPLV; ++c)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[c][e] += u * vr[c].get(e);
  };

  {
    // this wave's share of the block's active neurons: every NW-th one, starting at `wave`
    int total = 0;
    for (int w = 0; w < nwords; ++w) total += __popcll(uniform_u64(maskw[w]));
    const int mine = total > wave ? (total - wave + NW - 1) / NW : 0;
    Vec16<WT> ka[CPL2], va[CPLV], kb[CPL2], vb[CPLV];
    float sa, sb;
    int na = next_neuron();
    request(na, ka, va, sa);
    int nb = next_neuron();
    request(nb, kb, vb, sb);
    // The body is branch-free: a buffer whose neuron does not exist was requested through a
    // descriptor without records, holds zeros and adds zeros (only in the last round), so the
    // number of loads in flight is a compile-time constant and every wait is exact.
    for (int i = 0; i < mine; i += 2) {
      consume(na, ka, va, sa);
      na = next_neuron();
      request(na, ka, va, sa);
      consume(nb, kb, vb, sb);
      nb = next_neuron();
      request(nb, kb, vb, sb);
    }
  }

  // binary tree over the waves: in each round the upper half of the live waves hands its
  // row to the lower half through LDS
#pragma unroll
  for (int half = NW / 2; half >= 1; half >>= 1) {
    if (wave >= half && wave < 2 * half) {
      float* dst = rows + (size_t)(wave - half) * P.d_model;
#pragma unroll
      for (int c = 0; c < CPLV; ++c) {
        const int ch = lane + kWave * c;
        if (ch < nvecv) {
#pragma unroll
          for (int e = 0; e < VEC; e += 4)
            *reinterpret_cast<f32x4*>(dst + (size_t)ch * VEC + e) = f32x4{acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]};
        }
      }
    }
    __syncthreads();
    if (wave < half) {
      const float* src = rows + (size_t)wave * P.d_model;
#pragma unroll
      for (int c = 0; c < CPLV; ++c) {
        const int ch = lane + kWave * c;
        if (ch < nvecv) {
#pragma unroll
          for (int e = 0; e < VEC; e += 4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(src + (size_t)ch * VEC + e);
            acc[c][e] += t[0];
            acc[c][e + 1] += t[1];
            acc[c][e + 2] += t[2];
            acc[c][e + 3] += t[3];
          }
        }
      }
    }
    if (half > 1) __syncthreads();
  }
  if (wave == 0) {
    float* dst = P.part + ((size_t)l * P.NBC + blk) * P.d_model;
#pragma unroll
    for (int c = 0; c < CPLV; ++c) {
      const int ch = lane + kWave * c;
      if (ch < nvecv) {
#pragma unroll
        for (int e = 0; e < VEC; e += 4)
          *reinterpret_cast<f32x4*>(dst + (size_t)ch * VEC + e) = f32x4{acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]};
      }
    }
  }
}

// ---------------------------------------------------------------------------------- reduce
// y[l][c] = sum over the layer's gather blocks of part[l][blk][c].  Workgroup = 64 columns x 4
// slices of the blocks: a thread sums its slice in block order (16 loads in flight at a time), and
// the four slice sums of a column are added in slice order.
__global__ __launch_bounds__(256) void reduce_layers_kernel(const PhasedParams P) {
  constexpr int PER = 16;
  __shared__ float red[4][kWave];
  const int l = blockIdx.y, cg = threadIdx.x & (kWave - 1), sl = threadIdx.x / kWave;
  const int c = blockIdx.x * kWave + cg;
  const int per = (P.NBC + 3) / 4, b1 = min(P.NBC, (sl + 1) * per);
  const float* p = P.part + (size_t)l * P.NBC * P.d_model + (c < P.d_model ? c : 0);
  float acc = 0.f;
  for (int b0 = sl * per; b0 < b1; b0 += PER) {
    float t[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) t[i] = b0 + i < b1 ? p[(size_t)(b0 + i) * P.d_model] : 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) acc += t[i];
  }
  red[sl][cg] = acc;
  __syncthreads();
  if (sl == 0 && c < P.d_model) P.y[(size_t)l * P.d_model + c] = ((red[0][cg] + red[1][cg]) + red[2][cg]) + red[3][cg];
}

// ---------------------------------------------------------------------------------- select
// One workgroup per layer: count and ascending index list of {j : s_j > theta} (compaction by
// ballots and a running offset), with theta formed exactly as the gather workgroups form it.
__global__ __launch_bounds__(1024) void select_layers_kernel(const PhasedParams P) {
  __shared__ int wcount[16];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int l = blockIdx.x;
  const float theta = layer_theta(P, l, lane);
  int running = 0;
  for (int j0 = 0; j0 < P.d_ff; j0 += 1024) {
    const int j = j0 + tid;
    const bool on = j < P.d_ff && P.scores[(size_t)l * P.d_ff + j] > theta;
    const unsigned long long m = __ballot(on);
    if (lane == 0) wcount[wave] = __popcll(m);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      before += w < wave ? wcount[w] : 0;
      total += wcount[w];
    }
    if (on) {
      const int pos = running + before + lanes_below(m);
      if (P.idx) P.idx[(size_t)l * P.d_ff + pos] = j;
      if (P.uidx) P.uidx[(size_t)l * P.d_ff + pos] = j;
    }
    running += total;
    __syncthreads();
  }
  if (tid == 0) {
    if (P.count) P.count[l] = running;
    if (P.ucount) P.ucount[l] = running;
  }
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct PhasedLayout {
  size_t scores, stats, part, total;
};

// Scratch of a set of launches over up to `layer_cap` layers, with room for `part_rows` partial
// output rows in all.
PhasedLayout phased_layout(int d_model, int d_ff, int layer_cap, int part_rows) {
  PhasedLayout s;
  size_t o = 0;
  s.scores = o; o += align256((size_t)layer_cap * (size_t)d_ff * 4);
  s.stats = o;  o += align256((size_t)layer_cap * (size_t)((d_ff + 15) / 16) * 8);
  s.part = o;   o += align256((size_t)part_rows * (size_t)d_model * 4);
  s.total = o;
  return s;
}

// Compiled gather variants: chunks per lane of a K2n row and of a Vn row.
struct GatherVariant {
  int kind, cpl2, cplv, nw, occ;  // weight type (0 fp32, 1 bf16, 2 fp8, 3 int8), chunks, waves per workgroup,
                                  // waves per SIMD the registers are held to
};
constexpr GatherVariant kGather[] = {
    {1, 1, 1, 8, 4}, {1, 3, 5, 4, 3}, {1, 4, 7, 4, 2}, {0, 1, 1, 8, 4}, {0, 2, 2, 8, 4}, {0, 5, 9, 4, 2},
    {1, 3, 5, 8, 4},  // alternative for the 2B class (tuning switch)
    {2, 1, 1, 8, 4}, {2, 2, 3, 4, 3}, {2, 2, 4, 4, 2},
    {3, 1, 1, 8, 4}, {3, 2, 3, 4, 3}, {3, 2, 4, 4, 2},
};
constexpr int kNumGather = sizeof(kGather) / sizeof(kGather[0]);

int weight_kind(const FfnProblem& p) { return p.w_fp8 == 2 ? 3 : p.w_fp8 ? 2 : p.w_bf16 ? 1 : 0; }
int weight_vec(const FfnProblem& p) { return p.w_fp8 ? 16 : p.w_bf16 ? 8 : 4; }  // elements per 16 bytes

int gather_variant(const FfnProblem& p) {
  const int vec = weight_vec(p);
  const int c2 = ((p.d_model - p.r) / vec + kWave - 1) / kWave, cv = (p.d_model / vec + kWave - 1) / kWave;
  for (int i = 0; i < kNumGather; ++i)
    if (kGather[i].kind == weight_kind(p) && c2 <= kGather[i].cpl2 && cv <= kGather[i].cplv) return i;
  return -1;
}

template <typename WT, bool QB>
hipError_t launch_predict(const PhasedParams& P, int cpl1, dim3 grid, hipStream_t st) {
  if (P.RPB == 48 && cpl1 <= 2) {  // few layers: one sweep of 12 rows per wave
    if (cpl1 == 1) hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 1, 12>), grid, dim3(256), 0, st, P);
    else hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 2, 12>), grid, dim3(256), 0, st, P);
    return hipGetLastError();
  }
  switch (cpl1) {
    case 1: hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 1>), grid, dim3(256), 0, st, P); break;
    case 2: hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 2>), grid, dim3(256), 0, st, P); break;
    case 3: hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 3>), grid, dim3(256), 0, st, P); break;
    case 4: hipLaunchKernelGGL((predict_layers_kernel<WT, QB, 4>), grid, dim3(256), 0, st, P); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename WT, int CPL2, int CPLV, int NW, int OCC>
hipError_t launch_gather(const PhasedParams& P, dim3 grid, hipStream_t st) {
  constexpr int VEC = Vec16<WT>::N;
  // (at most 40 KB for the compiled variants: below the 64 KB a launch may ask for without an attribute)
  const size_t dyn = ((size_t)CPL2 * kWave * VEC + (size_t)(NW / 2) * P.d_model) * sizeof(float);
  hipLaunchKernelGGL((gather_layers_kernel<WT, CPL2, CPLV, NW, OCC>), grid, dim3(NW * kWave), dyn, st, P);
  return hipGetLastError();
}

template <int I>
hipError_t launch_gather_index(const PhasedParams& P, dim3 grid, hipStream_t st) {
  constexpr GatherVariant v = kGather[I];
  if constexpr (v.kind == 3) return launch_gather<i8_t, v.cpl2, v.cplv, v.nw, v.occ>(P, grid, st);
  else if constexpr (v.kind == 2) return launch_gather<fp8_t, v.cpl2, v.cplv, v.nw, v.occ>(P, grid, st);
  else if constexpr (v.kind == 1) return launch_gather<bf16_t, v.cpl2, v.cplv, v.nw, v.occ>(P, grid, st);
  else return launch_gather<float, v.cpl2, v.cplv, v.nw, v.occ>(P, grid, st);
}

}  // namespace

size_t phased_scratch_bytes(int d_model, int d_ff, int layer_cap) {
  return phased_layout(d_model, d_ff, layer_cap, layer_cap * kMaxNBC).total;
}

int phased_part_rows(size_t scratch_bytes, int d_model, int d_ff, int layer_cap) {
  const size_t fixed = phased_layout(d_model, d_ff, layer_cap, 0).total;
  if (scratch_bytes <= fixed) return 0;
  const size_t rows = (scratch_bytes - fixed) / ((size_t)d_model * 4);
  return (int)(rows < (size_t)layer_cap * kMostNBC ? rows : (size_t)layer_cap * kMostNBC);
}

bool phased_supported(const FfnProblem& p) {
  const int vec = weight_vec(p);
  const int c1 = (p.r / vec + kWave - 1) / kWave;
  const size_t lds = ((size_t)8 * kWave * 8 + (size_t)4 * p.d_model) * sizeof(float);
  return p.batch == 1 && c1 <= 4 && gather_variant(p) >= 0 && lds <= 150 * 1024;
}

hipError_t launch_ffn_phased(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                             const void* const* vn, int n_layers, int dense, const FfnTuning& tune, void* scratch,
                             int layer_cap, int part_rows, hipStream_t st) {
  layer_cap = max(1, min(layer_cap, kPhasedMaxLayers));
  if (part_rows < layer_cap) return hipErrorInvalidValue;
  const PhasedLayout lay = phased_layout(p0.d_model, p0.d_ff, layer_cap, part_rows);
  const int phases = (tune.phases & 7) ? (tune.phases & 7) : 7;
  int gv = gather_variant(p0);
  if (gv < 0) return hipErrorInvalidValue;
  if (gv == 1 && tune.variant == 1) gv = 6;
  const int vec = weight_vec(p0);
  const int cpl1 = (p0.r / vec + kWave - 1) / kWave;
  char* s = static_cast<char*>(scratch);
  hipError_t err = hipSuccess;
  for (int base = 0; base < n_layers && err == hipSuccess; base += layer_cap) {
    const int L = min(layer_cap, n_layers - base);
    PhasedParams P;
    for (int l = 0; l < kPhasedMaxLayers; ++l) {
      P.k1n[l] = l < L ? k1n[base + l] : nullptr;
      P.k2n[l] = l < L ? k2n[base + l] : nullptr;
      P.vn[l] = l < L ? vn[base + l] : nullptr;
    }
    P.q = p0.q;
    P.y = p0.y + (size_t)base * p0.d_model;
    P.theta = p0.theta ? p0.theta + base : nullptr;
    P.count = p0.active_count ? p0.active_count + base : nullptr;
    P.idx = p0.active_idx ? p0.active_idx + (size_t)base * p0.d_ff : nullptr;
    P.ucount = p0.union_count ? p0.union_count + base : nullptr;
    P.uidx = p0.union_idx ? p0.union_idx + (size_t)base * p0.d_ff : nullptr;
    P.scores = reinterpret_cast<float*>(s + lay.scores);
    P.stats = reinterpret_cast<float*>(s + lay.stats);
    P.part = reinterpret_cast<float*>(s + lay.part);
    P.n_layers = L;
    P.d_model = p0.d_model;
    P.d_ff = p0.d_ff;
    P.r = p0.r;
    P.q_bf16 = p0.q_bf16;
    P.gelu = p0.gelu;
    P.dense = dense;
    P.z = p0.z;
    // Block sizes: enough workgroups to fill 256 compute units several times over, as few
    // partial rows as that allows.
    const long long want_wg = 2048;
    int rpb = tune.rows_per_predict_block;
    if (rpb <= 0) {
      // 64 rows where that still gives every compute unit several workgroups; with fewer
      // layers 48 (measured best for 1..12 layers of the 2B shape: smaller blocks only lengthen
      // the list of block statistics every gather workgroup merges)
      rpb = (long long)L * ((p0.d_ff + 63) / 64) >= want_wg ? 64 : 48;
    }
    rpb = max(16, min(kMaxRPB, rpb / 16 * 16));
    int npb = tune.neurons_per_gather_block;
    if (npb <= 0) {
      // long per-wave runs of rows pipeline best: the largest block that still leaves about
      // two workgroups for every compute unit
      npb = 1024;
      while (npb > 64 && (long long)L * ((p0.d_ff + npb - 1) / npb) < 600) npb -= 64;
    }
    npb = max(64, min(1024, npb / 64 * 64));
    // partial rows: the scratch holds part_rows of them, shared by the L layers of this set
    const int nbc_cap = max(1, min(kMostNBC, part_rows / L));
    while ((p0.d_ff + npb - 1) / npb > nbc_cap) npb += 64;
    if (npb > 1024) return hipErrorInvalidValue;
    P.RPB = rpb;
    P.NBA = (p0.d_ff + rpb - 1) / rpb;
    P.NPB = npb;
    P.NBC = (p0.d_ff + npb - 1) / npb;

    const dim3 ga(P.NBA, L);
    if (!(phases & 1)) err = hipSuccess;
    else if (p0.w_fp8 == 2) err = launch_predict<i8_t, false>(P, cpl1, ga, st);
    else if (p0.w_fp8) err = launch_predict<fp8_t, false>(P, cpl1, ga, st);
    else if (p0.w_bf16) err = p0.q_bf16 ? launch_predict<bf16_t, true>(P, cpl1, ga, st) : launch_predict<bf16_t, false>(P, cpl1, ga, st);
    else err = launch_predict<float, false>(P, cpl1, ga, st);
    if (err != hipSuccess) return err;
    const dim3 gc(P.NBC, L);
    if (phases & 2) switch (gv) {
      case 0: err = launch_gather_index<0>(P, gc, st); break;
      case 1: err = launch_gather_index<1>(P, gc, st); break;
      case 2: err = launch_gather_index<2>(P, gc, st); break;
      case 3: err = launch_gather_index<3>(P, gc, st); break;
      case 4: err = launch_gather_index<4>(P, gc, st); break;
      case 5: err = launch_gather_index<5>(P, gc, st); break;
      case 6: err = launch_gather_index<6>(P, gc, st); break;
      case 7: err = launch_gather_index<7>(P, gc, st); break;
      case 8: err = launch_gather_index<8>(P, gc, st); break;
      case 9: err = launch_gather_index<9>(P, gc, st); break;
      case 10: err = launch_gather_index<10>(P, gc, st); break;
      case 11: err = launch_gather_index<11>(P, gc, st); break;
      case 12: err = launch_gather_index<12>(P, gc, st); break;
      default: err = hipErrorInvalidValue; break;
    }
    if (err != hipSuccess) return err;
    if (!(phases & 4)) continue;
    hipLaunchKernelGGL(reduce_layers_kernel, dim3((p0.d_model + kWave - 1) / kWave, L), dim3(256), 0, st, P);
    if (P.count || P.idx || P.ucount || P.uidx)
      hipLaunchKernelGGL(select_layers_kernel, dim3(L), dim3(1024), 0, st, P);
    err = hipGetLastError();
  }
  return err;
}

}  // namespace spark
