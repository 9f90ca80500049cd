// Spark-FFN decode (Eq.2 of arXiv 2506.06644), general path: any batch up to 64, any
// shape whose rows are multiples of 16 bytes.  Five launches per layer:
//   predict  S[b][j]   = K1n[j] . q_b[:r]                     (streams all of K1n once)
//   select   A[b][:]   = StatTop_k(S[b][:]), theta, idx, union flags   (stat_topk kernel)
//   union    U         = ascending compaction of the flags
//   k2       u[m][b]   = GELU(A[b][U[m]]) * (K2n[U[m]] . q_b[r:])      (reads only union rows)
//   v        y[b][c]   = sum_m u[m][b] * Vn[U[m]][c]                    (reads only union rows)
// Per-token masks skip arithmetic; the union decides which rows are fetched (Appendix B).
#include <algorithm>

#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

// 8-bit weight arrays carry one fp32 scale per row behind the last row of codes; other types none.
template <typename WT>
__device__ __forceinline__ float row_scale(const WT* w, int rows, int cols, int j) {
  if constexpr (sizeof(WT) == 1) return reinterpret_cast<const float*>(reinterpret_cast<const char*>(w) + (size_t)rows * (size_t)cols)[j];
  else return 1.f;
}
// two consecutive weights of a row (column c0 even) as floats
template <typename WT>
__device__ __forceinline__ void load_pair(const WT* p, float& w0, float& w1) {
  if constexpr (sizeof(WT) == 4) {
    const float2 w = *reinterpret_cast<const float2*>(p);
    w0 = w.x;
    w1 = w.y;
  } else if constexpr (sizeof(WT) == 2) {
    const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
    w0 = bf16_lo(w);
    w1 = bf16_hi(w);
  } else {
    Vec16<WT> v;
    v.raw = u32x4{(uint32_t)*reinterpret_cast<const uint16_t*>(p), 0u, 0u, 0u};
    w0 = v.get(0);
    w1 = v.get(1);
  }
}

// ---------------------------------------------------------------------------------- predict
template <typename WT, int TB>
__global__ __launch_bounds__(kBlock) void predict_kernel(const WT* __restrict__ k1n, int d_ff, int r,
                                                         const void* __restrict__ q, int q_bf16,
                                                         int64_t ldq, int B, float* __restrict__ S,
                                                         int32_t* __restrict__ flags) {
  constexpr int VEC = Vec16<WT>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  for (int i = blockIdx.x * kBlock + tid; i < d_ff; i += gridDim.x * kBlock) flags[i] = 0;
  const int nvec = r / VEC;
  const int gw = blockIdx.x * kWavesPerBlock + wave, nw = gridDim.x * kWavesPerBlock;
  for (int j = gw; j < d_ff; j += nw) {
    const WT* row = k1n + (int64_t)j * r;
    for (int b0 = 0; b0 < B; b0 += TB) {
      float acc[TB];
#pragma unroll
      for (int t = 0; t < TB; ++t) acc[t] = 0.f;
      for (int c = lane; c < nvec; c += kWave) {
        const Vec16<WT> w = load_vec16<WT>(row + (int64_t)c * VEC);
#pragma unroll
        for (int t = 0; t < TB; ++t) {
          if (b0 + t < B) {
            float qv[VEC];
            load_q_vec<VEC>(q, q_bf16, (int64_t)(b0 + t) * ldq + (int64_t)c * VEC, qv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[t] += w.get(e) * qv[e];
          }
        }
      }
#pragma unroll
      for (int t = 0; t < TB; ++t) {
        const float tot = wave_sum(acc[t]);
        if (lane == 0 && b0 + t < B) S[(int64_t)(b0 + t) * d_ff + j] = tot * row_scale<WT>(k1n, d_ff, r, j);
      }
    }
  }
}

// ---------------------------------------------------------------------------------- union
__global__ __launch_bounds__(1024) void union_kernel(const int32_t* __restrict__ flags, int d_ff,
                                                     int32_t* __restrict__ uidx,
                                                     int32_t* __restrict__ ucount,
                                                     int32_t* __restrict__ user_idx,
                                                     int32_t* __restrict__ user_count) {
  // One workgroup; thread t owns the consecutive entries [t * per, (t + 1) * per): counts,
  // one workgroup-wide exclusive scan of the counts, then ordered writes.
  constexpr int NW = 1024 / kWave;
  __shared__ int tab[NW];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int per = (d_ff + 1023) / 1024;
  const int lo = min(d_ff, tid * per), hi = min(d_ff, lo + per);
  int cnt = 0;
  for (int i = lo; i < hi; ++i) cnt += flags[i] != 0;
  int incl = cnt;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int t = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += t;
  }
  if (lane == kWave - 1) tab[wave] = incl;
  __syncthreads();
  int base = 0, total = 0;
  for (int w = 0; w < NW; ++w) {
    const int t = tab[w];
    if (w < wave) base += t;
    total += t;
  }
  int pos = base + incl - cnt;
  for (int i = lo; i < hi; ++i) {
    if (flags[i] != 0) {
      uidx[pos] = i;
      if (user_idx) user_idx[pos] = i;
      ++pos;
    }
  }
  if (tid == 0) {
    ucount[0] = total;
    if (user_count) user_count[0] = total;
  }
}

__global__ void iota_kernel(int d_ff, int32_t* __restrict__ uidx, int32_t* __restrict__ ucount) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < d_ff; i += gridDim.x * blockDim.x) uidx[i] = i;
  if (blockIdx.x == 0 && threadIdx.x == 0) ucount[0] = d_ff;
}

// ---------------------------------------------------------------------------------- k2
template <typename WT, int TB>
__global__ __launch_bounds__(kBlock) void k2_kernel(const WT* __restrict__ k2n, int d_ff, int r, int r2,
                                                    const void* __restrict__ q, int q_bf16, int64_t ldq,
                                                    int B, const float* __restrict__ A,
                                                    const int32_t* __restrict__ uidx,
                                                    const int32_t* __restrict__ ucount,
                                                    float* __restrict__ uact, int gelu_kind, int dense) {
  constexpr int VEC = Vec16<WT>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int nvec = r2 / VEC;
  const int m_total = ucount[0];
  const int gw = blockIdx.x * kWavesPerBlock + wave, nw = gridDim.x * kWavesPerBlock;
  for (int m = gw; m < m_total; m += nw) {
    const int j = uidx[m];
    const WT* row = k2n + (int64_t)j * r2;
    for (int b0 = 0; b0 < B; b0 += TB) {
      float a[TB], acc[TB];
      bool any = dense != 0;
#pragma unroll
      for (int t = 0; t < TB; ++t) {
        a[t] = (b0 + t < B) ? A[(int64_t)(b0 + t) * d_ff + j] : 0.f;
        any |= a[t] > 0.f;
        acc[t] = 0.f;
      }
      if (any) {
        for (int c = lane; c < nvec; c += kWave) {
          const Vec16<WT> w = load_vec16<WT>(row + (int64_t)c * VEC);
#pragma unroll
          for (int t = 0; t < TB; ++t) {
            if (b0 + t < B && (dense || a[t] > 0.f)) {
              float qv[VEC];
              load_q_vec<VEC>(q, q_bf16, (int64_t)(b0 + t) * ldq + r + (int64_t)c * VEC, qv);
#pragma unroll
              for (int e = 0; e < VEC; ++e) acc[t] += w.get(e) * qv[e];
            }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < TB; ++t) {
        const float g = any ? wave_sum(acc[t]) * row_scale<WT>(k2n, d_ff, r2, j) : 0.f;
        if (lane == 0 && b0 + t < B)
          uact[(int64_t)m * B + b0 + t] = a[t] > 0.f ? gelu(a[t], gelu_kind) * g : 0.f;
      }
    }
  }
}

// ---------------------------------------------------------------------------------- v
// Workgroup = 64 output columns x one slice of the union rows.  Thread t: column pair
// t % 32, row slot t / 32 (8 rows in flight per workgroup).
template <typename WT, int BT>
__global__ __launch_bounds__(kBlock) void v_kernel(const WT* __restrict__ vn, int d_ff, int d_model, int B,
                                                   const float* __restrict__ uact,
                                                   const int32_t* __restrict__ uidx,
                                                   const int32_t* __restrict__ ucount,
                                                   float* __restrict__ part) {
  constexpr int SLOTS = kBlock / 32;
  constexpr int CH = BT < 8 ? BT : 8;  // tokens reduced per LDS round
  __shared__ float red[SLOTS][CH][64];
  const int tid = threadIdx.x, cp = tid & 31, slot = tid >> 5;
  const int c0 = blockIdx.x * 64 + cp * 2;
  const bool col_ok = c0 < d_model;  // d_model is even
  const int m_total = ucount[0];
  const int ksplit = gridDim.y;
  const int per = (m_total + ksplit - 1) / ksplit;
  const int m_lo = blockIdx.y * per;
  const int m_hi = min(m_total, m_lo + per);

  float acc[BT][2];
#pragma unroll
  for (int b = 0; b < BT; ++b) acc[b][0] = acc[b][1] = 0.f;

  if (col_ok) {
    for (int m = m_lo + slot; m < m_hi; m += SLOTS) {
      const int j = uidx[m];
      const WT* p = vn + (int64_t)j * d_model + c0;
      float w0, w1;
      load_pair<WT>(p, w0, w1);
      const float sv = row_scale<WT>(vn, d_ff, d_model, j);
      const float* up = uact + (int64_t)m * B;
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        if (b < B) {
          const float u = up[b] * sv;
          acc[b][0] += u * w0;
          acc[b][1] += u * w1;
        }
      }
    }
  }

  // combine the 8 row slots, CH tokens per round
#pragma unroll
  for (int b0 = 0; b0 < BT; b0 += CH) {
    if (b0 >= B) break;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < CH; ++t) {
      red[slot][t][cp * 2] = acc[b0 + t][0];
      red[slot][t][cp * 2 + 1] = acc[b0 + t][1];
    }
    __syncthreads();
    for (int o = tid; o < CH * 64; o += kBlock) {
      const int t = o >> 6, c = o & 63;
      float s = 0.f;
#pragma unroll
      for (int sl = 0; sl < SLOTS; ++sl) s += red[sl][t][c];
      const int b = b0 + t, col = blockIdx.x * 64 + c;
      if (b < B && col < d_model) part[((int64_t)blockIdx.y * B + b) * d_model + col] = s;
    }
  }
}

__global__ __launch_bounds__(kBlock) void reduce_kernel(const float* __restrict__ part, int ksplit,
                                                        int64_t n, float* __restrict__ y) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  // slices are added in ascending order; the loads of eight slices are issued together
  float s = 0.f;
  int ks = 0;
  for (; ks + 8 <= ksplit; ks += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(ks + u) * n + i];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; ks < ksplit; ++ks) s += part[(int64_t)ks * n + i];
  y[i] = s;
}

// ------------------------------------------------------------------- batched path on MFMA
// For batches of 2..64 tokens with bf16 weights and bf16 tokens the two row-times-token
// products are small GEMMs (Appendix B: the prefill / chunk case):
//   rows x tokens:   G[j][b] = W[j][:] . q_b[off : off + K]   for 16 rows j and all tokens
// v_mfma_f32_16x16x32_bf16 takes, per lane, 8 consecutive k of one row (A) and 8 consecutive
// k of one token (B): both are plain 16-byte loads of the neuron-major / token-major arrays.
// bf16 x bf16 products are exact in fp32 and the accumulation is fp32, as in the batch-1 path.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// One workgroup (8 waves) = one tile of 16 rows; the waves take every 8th step of 32 k (so that
// for r around 1024 a wave issues all its loads at once) and their partial tiles are summed
// through LDS in wave order.  MODE 0: rows are neurons
// 16 * tile + i and the result goes to S[b][j].  MODE 1: rows are union entries
// uidx[16 * tile + i] and the result becomes uact[m][b] = GELU(A[b][j]) * g (0 if A[b][j] <= 0).
constexpr int kRowsWaves = 8;
template <int NB, int MODE>
__global__ __launch_bounds__(kRowsWaves * kWave) void rows_mfma_kernel(const bf16_t* __restrict__ w, int n_rows, int K,
                                                        const bf16_t* __restrict__ q, int64_t ldq, int qoff,
                                                        int B, int d_ff, const int32_t* __restrict__ uidx,
                                                        const int32_t* __restrict__ ucount,
                                                        const float* __restrict__ A, float* __restrict__ out,
                                                        int gelu_kind, int dense, int32_t* __restrict__ flags) {
  __shared__ float red[kRowsWaves - 1][NB * 4][kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int tile = blockIdx.x;
  if (MODE == 0) {
    for (int i = blockIdx.x * blockDim.x + tid; i < d_ff; i += gridDim.x * blockDim.x) flags[i] = 0;
  }
  const int m_total = MODE == 0 ? n_rows : ucount[0];
  if (tile * 16 >= m_total) return;
  const int ri = lane & 15, kg = lane >> 4;  // row (or token) within the tile, group of 8 k
  const int m = tile * 16 + ri;
  const int mc = m < m_total ? m : m_total - 1;
  const int j = MODE == 0 ? mc : uidx[mc];
  const bf16_t* wrow = w + (int64_t)j * K;
  const bf16_t* qrow[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int b = nb * 16 + ri;
    qrow[nb] = q + (int64_t)(b < B ? b : B - 1) * ldq + qoff;
  }
  const int nchunk = K / 8;               // 16-byte chunks per row
  const int nsteps = (nchunk + 3) / 4;    // steps of 32 k
  f32x4 acc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = wave; s0 < nsteps; s0 += 4 * kRowsWaves) {
    u32x4 a[4], bq[4][NB];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ch = (s0 + kRowsWaves * u) * 4 + kg;
      const bool ok = s0 + kRowsWaves * u < nsteps && ch < nchunk;
      const int chc = ok ? ch : 0;
      a[u] = *reinterpret_cast<const u32x4*>(wrow + (int64_t)chc * 8);
      if (!ok) a[u] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bq[u][nb] = *reinterpret_cast<const u32x4*>(qrow[nb] + (int64_t)chc * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[u]),
                                                          __builtin_bit_cast(bf16x8_t, bq[u][nb]), acc[nb], 0, 0, 0);
  }
  // sum the waves' tiles in wave order
  if (wave > 0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 4; ++e) red[wave - 1][nb * 4 + e][lane] = acc[nb][e];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
      for (int wv = 0; wv < kRowsWaves - 1; ++wv) acc[nb][e] += red[wv][nb * 4 + e][lane];
    }
  // lane holds D[row 4 * kg + e][token ri] of every token block
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int b = nb * 16 + ri;
    if (b >= B) continue;
    if (MODE == 0 && (d_ff & 3) == 0 && tile * 16 + 4 * kg + 3 < m_total) {
      *reinterpret_cast<f32x4*>(out + (int64_t)b * d_ff + tile * 16 + 4 * kg) = acc[nb];
      continue;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int mm = tile * 16 + 4 * kg + e;
      if (mm >= m_total) continue;
      if (MODE == 0) {
        out[(int64_t)b * d_ff + mm] = acc[nb][e];
      } else {
        const int jj = uidx[mm];
        const float av = A[(int64_t)b * d_ff + jj];
        out[(int64_t)mm * B + b] = av > 0.f ? gelu(av, gelu_kind) * acc[nb][e] : 0.f;
      }
    }
  }
}

// y partials: part[ks][b][c] = sum over the union rows m of slice ks of uact[m][b] * Vn[U[m]][c].
// The contraction runs over rows while Vn is contiguous along columns, so the bf16 MFMA
// (which wants 8 consecutive k per lane) would need a transpose; v_mfma_f32_32x32x2_f32 takes a
// single k per lane instead: lanes 0..31 hold one row and lanes 32..63 the next, each lane
// two columns (one 4-byte load, 128 bytes per row and wave), widened to fp32.  A = uact
// (32 tokens x 2 rows), D = 32 tokens x 32 columns, two column phases, NH token halves.
// The loop is software-pipelined by hand: row indices are fetched two steps ahead and the
// rows themselves one step ahead of the MFMAs that consume them.
template <int NH>
__global__ __launch_bounds__(256) void v_mfma_kernel(const bf16_t* __restrict__ vn, int d_model, int B,
                                                     const float* __restrict__ uact,
                                                     const int32_t* __restrict__ uidx,
                                                     const int32_t* __restrict__ ucount,
                                                     float* __restrict__ part) {
  extern __shared__ float vred[];  // [NH * 32][kWave]
  constexpr int UNR = 8;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int half = lane >> 5, cl = lane & 31;
  const int c0 = blockIdx.x * 64 + cl * 2;
  const bool col_ok = c0 < d_model;
  const int cc = col_ok ? c0 : 0;
  const int m_total = ucount[0];
  const int ksplit = gridDim.y;
  const int per = ((m_total + ksplit - 1) / ksplit + 1) / 2 * 2;  // even: rows are taken in pairs
  const int m_lo = blockIdx.y * per;
  const int m_hi = min(m_total, m_lo + per);
  const int m_safe = m_total > 0 ? min(m_lo, m_total - 1) : 0;  // a valid row for clamped reads

  f32x16 acc[NH][2];
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int x = 0; x < 16; ++x) acc[h][e][x] = 0.f;

  // row of (step t, slot u) for this lane; rows past the slice are clamped and weighted by 0
  auto row_of = [&](int t, int u) { return m_lo + 2 * wave + half + 8 * (t * UNR + u); };
  auto load_j = [&](int t, int (&j)[UNR]) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int m = row_of(t, u);
      j[u] = uidx[m < m_hi ? m : m_safe];
    }
  };
  auto load_rows = [&](int t, const int (&j)[UNR], uint32_t (&vv)[UNR], float (&av)[UNR][NH]) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int m = row_of(t, u);
      const bool ok = m < m_hi;
      vv[u] = *reinterpret_cast<const uint32_t*>(vn + (int64_t)j[u] * d_model + cc);
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const int b = 32 * h + cl;
        const float a = uact[(int64_t)(ok ? m : m_safe) * B + (b < B ? b : 0)];
        av[u][h] = (ok && b < B) ? a : 0.f;
      }
    }
  };
  const int rows_w = max(0, m_hi - (m_lo + 2 * wave));      // rows from this wave's first pair on
  const int steps = (rows_w + 8 * UNR - 1) / (8 * UNR);
  if (m_total > 0 && steps > 0) {
    int j0[UNR], j1[UNR];
    uint32_t v0[UNR], v1[UNR];
    float a0[UNR][NH], a1[UNR][NH];
    load_j(0, j0);
    load_j(1, j1);
    load_rows(0, j0, v0, a0);
    for (int t = 0; t < steps; ++t) {
      int j2[UNR];
      load_j(t + 2, j2);
      load_rows(t + 1, j1, v1, a1);
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const float w[2] = {bf16_lo(v0[u]), bf16_hi(v0[u])};
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
          for (int e = 0; e < 2; ++e) acc[h][e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u][h], w[e], acc[h][e], 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        v0[u] = v1[u];
        j1[u] = j2[u];
#pragma unroll
        for (int h = 0; h < NH; ++h) a0[u][h] = a1[u][h];
      }
    }
  }
  // sum the four waves' tiles through LDS in wave order, then wave 0 stores
  for (int wv = 3; wv >= 1; --wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            float* slot = &vred[((h * 2 + e) * 16 + x) * kWave + lane];
            *slot = (wv == 3) ? acc[h][e][x] : *slot + acc[h][e][x];
          }
    }
  }
  __syncthreads();
  if (wave != 0 || !col_ok) return;
  float* dst = part + (int64_t)blockIdx.y * B * d_model;
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      // D[i][n]: n = lane % 32, i = 8 * (x / 4) + 4 * (lane / 32) + x % 4
      const int b = 32 * h + 8 * (x / 4) + 4 * half + (x % 4);
      if (b >= B) continue;
      float2 o;
      o.x = acc[h][0][x] + vred[((h * 2 + 0) * 16 + x) * kWave + lane];
      o.y = acc[h][1][x] + vred[((h * 2 + 1) * 16 + x) * kWave + lane];
      *reinterpret_cast<float2*>(dst + (int64_t)b * d_model + c0) = o;
    }
}

// ------------------------------------------------------------------- dense comparison path
// Batch 1, every neuron's K2n and Vn row is read (Eq.3 instead of Eq.4): the same-GPU
// comparison point of the sparse path.  Three launches: all scores and all K2 products in one
// sweep over K1n and K2n, the statistical top-k of the scores, a column-blocked sweep over Vn.
template <typename WT>
__global__ __launch_bounds__(256) void dense_rows_kernel(const WT* __restrict__ k1n, const WT* __restrict__ k2n,
                                                         int d_ff, int r, int r2, const void* __restrict__ q,
                                                         int q_bf16, float* __restrict__ S, float* __restrict__ G,
                                                         int32_t* __restrict__ flags) {
  constexpr int VEC = Vec16<WT>::N;
  extern __shared__ float qs[];  // q as fp32, d_model entries
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  for (int i = blockIdx.x * 256 + tid; i < d_ff; i += gridDim.x * 256) flags[i] = 0;
  for (int i = tid; i < r + r2; i += 256) qs[i] = load_q(q, q_bf16, i);
  __syncthreads();
  const int nvec1 = r / VEC, nvec2 = r2 / VEC;
  const int gw = blockIdx.x * 4 + wave, nw = gridDim.x * 4;
  for (int j = gw * 2; j < d_ff; j += nw * 2) {
    const int jb = j + 1 < d_ff ? j + 1 : j;
    const WT *a1 = k1n + (int64_t)j * r, *b1 = k1n + (int64_t)jb * r;
    const WT *a2 = k2n + (int64_t)j * r2, *b2 = k2n + (int64_t)jb * r2;
    float sa = 0.f, sb = 0.f, ga = 0.f, gb = 0.f;
    for (int c = lane; c < nvec1; c += kWave) {
      const Vec16<WT> wa = load_vec16<WT>(a1 + (int64_t)c * VEC), wb = load_vec16<WT>(b1 + (int64_t)c * VEC);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float qv = qs[c * VEC + e];
        sa += wa.get(e) * qv;
        sb += wb.get(e) * qv;
      }
    }
    for (int c = lane; c < nvec2; c += kWave) {
      const Vec16<WT> wa = load_vec16<WT>(a2 + (int64_t)c * VEC), wb = load_vec16<WT>(b2 + (int64_t)c * VEC);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float qv = qs[r + c * VEC + e];
        ga += wa.get(e) * qv;
        gb += wb.get(e) * qv;
      }
    }
    sa = wave_sum(sa);
    sb = wave_sum(sb);
    ga = wave_sum(ga);
    gb = wave_sum(gb);
    if (lane == 0) {
      S[j] = sa;
      G[j] = ga;
      if (j + 1 < d_ff) {
        S[j + 1] = sb;
        G[j + 1] = gb;
      }
    }
  }
}

// part[ks][c] = sum over the rows j of slice ks of u_j * Vn[j][c], u_j = GELU(a_j) * g_j (0 where
// a_j <= 0).  Thread = (16-byte column chunk cc of 16, row group rr of 32); the 32 row groups
// are summed through LDS in a fixed order.
template <typename WT>
__global__ __launch_bounds__(512) void dense_v_kernel(const WT* __restrict__ vn, int d_ff, int d_model,
                                                      const float* __restrict__ A, const float* __restrict__ G,
                                                      int gelu_kind, float* __restrict__ part) {
  constexpr int VEC = Vec16<WT>::N;
  constexpr int RG = 32, UNR = 4;
  __shared__ float red[RG][16 * VEC + 1];
  const int tid = threadIdx.x, cc = tid & 15, rr = tid >> 4;
  const int col0 = (blockIdx.x * 16 + cc) * VEC;
  const bool col_ok = col0 < d_model;
  const int per = (d_ff + gridDim.y - 1) / gridDim.y;
  const int j_lo = blockIdx.y * per, j_hi = min(d_ff, j_lo + per);
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  for (int j0 = j_lo + rr; j0 < j_hi; j0 += RG * UNR) {
    Vec16<WT> w[UNR];
    float u[UNR];
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int j = j0 + RG * t;
      const bool ok = j < j_hi;
      const int jc = ok ? j : j_lo;
      w[t] = load_vec16<WT>(vn + (int64_t)jc * d_model + (col_ok ? col0 : 0));
      const float a = A[jc];
      u[t] = (ok && a > 0.f) ? gelu(a, gelu_kind) * G[jc] : 0.f;
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += u[t] * w[t].get(e);
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) red[rr][cc * VEC + e] = acc[e];
  __syncthreads();
  if (tid < 16 * VEC) {
    float s = 0.f;
    for (int g = 0; g < RG; ++g) s += red[g][tid];
    const int c = blockIdx.x * 16 * VEC + tid;
    if (c < d_model) part[(int64_t)blockIdx.y * d_model + c] = s;
  }
}

template <typename WT>
hipError_t launch_general_t(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st) {
  const WT* k1n = static_cast<const WT*>(p.k1n);
  const WT* k2n = static_cast<const WT*>(p.k2n);
  const WT* vn = static_cast<const WT*>(p.vn);
  const int B = p.batch;
  const int r2 = p.d_model - p.r;

  if constexpr (sizeof(WT) == 1) {
    if (dense) return hipErrorInvalidValue;  // (8-bit weights: the dense comparison exists on the one-token path only)
  }
  if (dense && B == 1) {
    hipLaunchKernelGGL((dense_rows_kernel<WT>), dim3(2048), dim3(256), (size_t)p.d_model * 4, st, k1n, k2n, p.d_ff,
                       p.r, r2, p.q, p.q_bf16, ws.S, ws.uact, ws.flags);
    hipError_t e = launch_stat_topk(ws.S, 0, 1, p.d_ff, p.d_ff, p.z, 0, 0.f, ws.A, p.d_ff, p.theta, p.active_count,
                                    p.active_idx, p.d_ff, nullptr, st);
    if (e != hipSuccess) return e;
    constexpr int VEC = Vec16<WT>::N;
    const dim3 grid((p.d_model + 16 * VEC - 1) / (16 * VEC), ws.ksplit);
    hipLaunchKernelGGL((dense_v_kernel<WT>), grid, dim3(512), 0, st, vn, p.d_ff, p.d_model, ws.A, ws.uact, p.gelu,
                       ws.part);
    hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((p.d_model + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                       ws.part, ws.ksplit, (int64_t)p.d_model, p.y);
    return hipGetLastError();
  }

  if constexpr (sizeof(WT) == 2) {
    if (B >= 2 && p.q_bf16) {
      const bf16_t* qb = static_cast<const bf16_t*>(p.q);
      const int tiles = (p.d_ff + 15) / 16;
      const int nb = (B + 15) / 16;
#define SPARK_LAUNCH_ROWS(NB, MODE, W, K, QOFF, OUT)                                                     \
  hipLaunchKernelGGL((rows_mfma_kernel<NB, MODE>), dim3(tiles), dim3(kRowsWaves * kWave), 0, st, W, p.d_ff, K, qb, p.ldq, \
                     QOFF, B, p.d_ff, ws.uidx, ws.ucount, ws.A, OUT, p.gelu, dense, ws.flags)
      if (nb == 1) SPARK_LAUNCH_ROWS(1, 0, k1n, p.r, 0, ws.S);
      else if (nb == 2) SPARK_LAUNCH_ROWS(2, 0, k1n, p.r, 0, ws.S);
      else SPARK_LAUNCH_ROWS(4, 0, k1n, p.r, 0, ws.S);
      hipError_t e = launch_stat_topk(ws.S, 0, B, p.d_ff, p.d_ff, p.z, 0, 0.f, ws.A, p.d_ff, p.theta, p.active_count,
                                      p.active_idx, p.d_ff, ws.flags, st);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(union_kernel, dim3(1), dim3(1024), 0, st, ws.flags, p.d_ff, ws.uidx, ws.ucount,
                         p.union_idx, p.union_count);
      if (dense) hipLaunchKernelGGL(iota_kernel, dim3(16), dim3(256), 0, st, p.d_ff, ws.uidx, ws.ucount);
      if (nb == 1) SPARK_LAUNCH_ROWS(1, 1, k2n, r2, p.r, ws.uact);
      else if (nb == 2) SPARK_LAUNCH_ROWS(2, 1, k2n, r2, p.r, ws.uact);
      else SPARK_LAUNCH_ROWS(4, 1, k2n, r2, p.r, ws.uact);
#undef SPARK_LAUNCH_ROWS
      const int ksv = ws.ksplit < 16 ? ws.ksplit : 16;
      const dim3 vgrid((p.d_model + 63) / 64, ksv);
      if (B <= 32)
        hipLaunchKernelGGL((v_mfma_kernel<1>), vgrid, dim3(256), 32 * kWave * 4, st, vn, p.d_model, B, ws.uact,
                           ws.uidx, ws.ucount, ws.part);
      else
        hipLaunchKernelGGL((v_mfma_kernel<2>), vgrid, dim3(256), 2 * 32 * kWave * 4, st, vn, p.d_model, B,
                           ws.uact, ws.uidx, ws.ucount, ws.part);
      const int64_t n = (int64_t)B * p.d_model;
      hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, ws.part,
                         ksv, n, p.y);
      return hipGetLastError();
    }
  }

  {
    const int grid = min((p.d_ff + kWavesPerBlock - 1) / kWavesPerBlock, 4096);
    if (B == 1)
      hipLaunchKernelGGL((predict_kernel<WT, 1>), dim3(grid), dim3(kBlock), 0, st, k1n, p.d_ff, p.r, p.q,
                         p.q_bf16, p.ldq, B, ws.S, ws.flags);
    else
      hipLaunchKernelGGL((predict_kernel<WT, 4>), dim3(grid), dim3(kBlock), 0, st, k1n, p.d_ff, p.r, p.q,
                         p.q_bf16, p.ldq, B, ws.S, ws.flags);
  }
  hipError_t e = launch_stat_topk(ws.S, 0, B, p.d_ff, p.d_ff, p.z, 0, 0.f, ws.A, p.d_ff, p.theta, p.active_count,
                                  p.active_idx, p.d_ff, ws.flags, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(union_kernel, dim3(1), dim3(1024), 0, st, ws.flags, p.d_ff, ws.uidx, ws.ucount,
                     p.union_idx, p.union_count);
  if (dense) hipLaunchKernelGGL(iota_kernel, dim3(16), dim3(256), 0, st, p.d_ff, ws.uidx, ws.ucount);
  {
    const int grid = dense ? 2048 : 512;
    if (B == 1)
      hipLaunchKernelGGL((k2_kernel<WT, 1>), dim3(grid), dim3(kBlock), 0, st, k2n, p.d_ff, p.r, r2, p.q,
                         p.q_bf16, p.ldq, B, ws.A, ws.uidx, ws.ucount, ws.uact, p.gelu, dense);
    else
      hipLaunchKernelGGL((k2_kernel<WT, 4>), dim3(grid), dim3(kBlock), 0, st, k2n, p.d_ff, p.r, r2, p.q,
                         p.q_bf16, p.ldq, B, ws.A, ws.uidx, ws.ucount, ws.uact, p.gelu, dense);
  }
  {
    const dim3 grid((p.d_model + 63) / 64, ws.ksplit);
    float* out = ws.ksplit == 1 ? p.y : ws.part;
#define SPARK_LAUNCH_V(BT)                                                                          \
  hipLaunchKernelGGL((v_kernel<WT, BT>), grid, dim3(kBlock), 0, st, vn, p.d_ff, p.d_model, B, ws.uact, ws.uidx, \
                     ws.ucount, out)
    if (B == 1) SPARK_LAUNCH_V(1);
    else if (B <= 4) SPARK_LAUNCH_V(4);
    else if (B <= 16) SPARK_LAUNCH_V(16);
    else SPARK_LAUNCH_V(64);
#undef SPARK_LAUNCH_V
    if (ws.ksplit > 1) {
      const int64_t n = (int64_t)B * p.d_model;
      hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                         ws.part, ws.ksplit, n, p.y);
    }
  }
  return hipGetLastError();
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int pick_ksplit(int d_model) {
  const int col_tiles = (d_model + 63) / 64;
  int ks = (1024 + col_tiles - 1) / col_tiles;
  if (ks > 32) ks = 32;
  if (ks < 1) ks = 1;
  return ks;
}


}  // namespace

// The region the phase-by-phase paths use (one of them runs per call).
static size_t phased_region_bytes(int d_model, int d_ff, int batch) {
  if (batch >= 2) return phased_batch_scratch_bytes(d_model, d_ff, batch);
  return phased_scratch_bytes(d_model, d_ff, kPhasedMaxLayers);
}

size_t ffn_workspace_bytes(int d_model, int d_ff, int batch) {
  const size_t B = (size_t)batch, F = (size_t)d_ff, D = (size_t)d_model;
  size_t t = 0;
  t += align_up(B * F * 4, 256);                       // S
  t += align_up(B * F * 4, 256);                       // A
  t += align_up(F * 4, 256);                           // flags
  t += align_up(F * 4, 256);                           // uidx
  t += 256;                                            // ucount
  t += align_up(F * B * 4, 256);                       // uact
  t += align_up((size_t)pick_ksplit(d_model) * B * D * 4, 256);  // part
  t += align_up(phased_region_bytes(d_model, d_ff, batch), 256);
  return t;
}

FfnWorkspace carve_workspace(void* base, int d_model, int d_ff, int batch) {
  const size_t B = (size_t)batch, F = (size_t)d_ff, D = (size_t)d_model;
  char* p = static_cast<char*>(base);
  FfnWorkspace ws;
  ws.S = reinterpret_cast<float*>(p);        p += align_up(B * F * 4, 256);
  ws.A = reinterpret_cast<float*>(p);        p += align_up(B * F * 4, 256);
  ws.flags = reinterpret_cast<int32_t*>(p);  p += align_up(F * 4, 256);
  ws.uidx = reinterpret_cast<int32_t*>(p);   p += align_up(F * 4, 256);
  ws.ucount = reinterpret_cast<int32_t*>(p); p += 256;
  ws.uact = reinterpret_cast<float*>(p);     p += align_up(F * B * 4, 256);
  ws.ksplit = pick_ksplit(d_model);
  ws.part = reinterpret_cast<float*>(p);     p += align_up((size_t)ws.ksplit * B * D * 4, 256);
  ws.phased = p;
  ws.phased_bytes = phased_region_bytes(d_model, d_ff, batch);
  return ws;
}

hipError_t launch_ffn_general(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st) {
  if (p.w_fp8 == 2) return launch_general_t<i8_t>(p, ws, dense, st);
  if (p.w_fp8) return launch_general_t<fp8_t>(p, ws, dense, st);
  return p.w_bf16 ? launch_general_t<bf16_t>(p, ws, dense, st) : launch_general_t<float>(p, ws, dense, st);
}

}  // namespace spark
