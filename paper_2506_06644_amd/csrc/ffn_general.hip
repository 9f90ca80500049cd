// Spark-FFN decode (Eq.2 of arXiv 2506.06644), general path: any batch up to 64, any
// shape whose rows are multiples of 16 bytes.  Five launches per layer:
//   predict  S[b][j]   = K1n[j] . q_b[:r]                     (streams all of K1n once)
//   select   A[b][:]   = StatTop_k(S[b][:]), theta, idx, union flags   (stat_topk kernel)
//   union    U         = ascending compaction of the flags
//   k2       u[m][b]   = GELU(A[b][U[m]]) * (K2n[U[m]] . q_b[r:])      (reads only union rows)
//   v        y[b][c]   = sum_m u[m][b] * Vn[U[m]][c]                    (reads only union rows)
// Per-token masks skip arithmetic; the union decides which rows are fetched (Appendix B).
#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

// ---------------------------------------------------------------------------------- predict
template <typename WT, int TB>
__global__ __launch_bounds__(kBlock) void predict_kernel(const WT* __restrict__ k1n, int d_ff, int r,
                                                         const void* __restrict__ q, int q_bf16,
                                                         int64_t ldq, int B, float* __restrict__ S,
                                                         int32_t* __restrict__ flags,
                                                         int32_t* __restrict__ status) {
  constexpr int VEC = Vec16<WT>::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  for (int i = blockIdx.x * kBlock + tid; i < d_ff; i += gridDim.x * kBlock) flags[i] = 0;
  if (blockIdx.x == 0 && tid == 0) status[0] = 0;  // this path cannot abort
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
        if (lane == 0 && b0 + t < B) S[(int64_t)(b0 + t) * d_ff + j] = tot;
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
  constexpr int NW = 1024 / kWave;
  __shared__ int tab[NW];
  __shared__ int running;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  if (tid == 0) running = 0;
  __syncthreads();
  for (int base = 0; base < d_ff; base += 1024) {
    const int i = base + tid;
    const bool a = i < d_ff && flags[i] != 0;
    const uint64_t b = __ballot(a);
    if (lane == 0) tab[wave] = __popcll(b);
    __syncthreads();
    int pos = running + lanes_below(b);
    for (int w = 0; w < wave; ++w) pos += tab[w];
    if (a) {
      uidx[pos] = i;
      if (user_idx) user_idx[pos] = i;
    }
    __syncthreads();
    if (tid == 0) {
      int t = running;
      for (int w = 0; w < NW; ++w) t += tab[w];
      running = t;
    }
    __syncthreads();
  }
  if (tid == 0) {
    ucount[0] = running;
    if (user_count) user_count[0] = running;
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
        const float g = any ? wave_sum(acc[t]) : 0.f;
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
__global__ __launch_bounds__(kBlock) void v_kernel(const WT* __restrict__ vn, int d_model, int B,
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
      if (sizeof(WT) == 2) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        w0 = bf16_lo(w);
        w1 = bf16_hi(w);
      } else {
        const float2 w = *reinterpret_cast<const float2*>(p);
        w0 = w.x;
        w1 = w.y;
      }
      const float* up = uact + (int64_t)m * B;
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        if (b < B) {
          const float u = up[b];
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
  float s = 0.f;
  for (int ks = 0; ks < ksplit; ++ks) s += part[(int64_t)ks * n + i];
  y[i] = s;
}

template <typename WT>
hipError_t launch_general_t(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st) {
  const WT* k1n = static_cast<const WT*>(p.k1n);
  const WT* k2n = static_cast<const WT*>(p.k2n);
  const WT* vn = static_cast<const WT*>(p.vn);
  const int B = p.batch;
  const int r2 = p.d_model - p.r;

  {
    const int grid = min((p.d_ff + kWavesPerBlock - 1) / kWavesPerBlock, 4096);
    if (B == 1)
      hipLaunchKernelGGL((predict_kernel<WT, 1>), dim3(grid), dim3(kBlock), 0, st, k1n, p.d_ff, p.r, p.q,
                         p.q_bf16, p.ldq, B, ws.S, ws.flags, static_cast<int32_t*>(ws.fused));
    else
      hipLaunchKernelGGL((predict_kernel<WT, 4>), dim3(grid), dim3(kBlock), 0, st, k1n, p.d_ff, p.r, p.q,
                         p.q_bf16, p.ldq, B, ws.S, ws.flags, static_cast<int32_t*>(ws.fused));
  }
  hipError_t e = launch_stat_topk(ws.S, 0, B, p.d_ff, p.d_ff, p.z, 0, ws.A, p.d_ff, p.theta, p.active_count,
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
  hipLaunchKernelGGL((v_kernel<WT, BT>), grid, dim3(kBlock), 0, st, vn, p.d_model, B, ws.uact, ws.uidx, \
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
  t += align_up(fused_scratch_bytes(d_model, d_ff), 256);
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
  ws.fused = p;
  ws.fused_bytes = fused_scratch_bytes(d_model, d_ff);
  return ws;
}

hipError_t launch_ffn_general(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st) {
  return p.w_bf16 ? launch_general_t<bf16_t>(p, ws, dense, st) : launch_general_t<float>(p, ws, dense, st);
}

}  // namespace spark
