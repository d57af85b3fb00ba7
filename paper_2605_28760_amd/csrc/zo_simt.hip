// fp32 kernels on the vector ALU: the same probe linear (Sec. 3.2) and fused
// head scoring (Sec. 3.3) as the matrix-core path, for fp32 operands.  They
// exist for the small fp32 configuration where results must agree with an
// fp64 reference to ~1e-5; they are simple LDS-tiled SIMT GEMMs.
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

constexpr int ST = kSimtTile;  // 64x64 output tile, 16-deep K slab, 4x4 per thread
constexpr int SK = 16;

// Tside[t, :] = [ s_t eps X[t,:] V_{k_t} | X[t,:] Vb ]; zero where the row has no such term.
__global__ void k_side_f32(ProbeF32Args p) {
  const int NC = p.r + p.R;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)p.T * NC) return;
  const int t = (int)(idx / NC), j = (int)(idx % NC);
  const int s = p.tok_seq[t];
  const int kind = p.seq_kind[s];
  float acc = 0.0f;
  const float* x = p.X + (int64_t)t * p.ldx;
  if (j < p.r) {
    if (kind >= 0) {
      const float* v = p.Vf + (int64_t)kind * p.n * p.r + j;
      for (int i = 0; i < p.n; ++i) acc = fmaf(x[i], v[(int64_t)i * p.r], acc);
      acc *= p.seq_scale[s];
    }
  } else if (kind >= kKindCentre) {
    const float* v = p.Vb + (j - p.r);
    for (int i = 0; i < p.n; ++i) acc = fmaf(x[i], v[(int64_t)i * p.R_cap], acc);
  }
  p.Tside[idx] = acc;
}

// acc[i][j] = sum_k A[m0 + ty*4 + i][k] * B[n0 + tx*4 + j][k]
__device__ __forceinline__ void simt_mainloop(const float* __restrict__ A, int64_t lda, int M, int m0,
                                              const float* __restrict__ B, int64_t ldb, int N, int n0,
                                              int K, float (&acc)[4][4]) {
  __shared__ float As[SK][ST + 1];
  __shared__ float Bs[SK][ST + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  for (int k0 = 0; k0 < K; k0 += SK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = tid + e * 256;
      const int row = idx >> 4, kk = idx & 15;
      const bool kin = k0 + kk < K;
      As[kk][row] = (kin && m0 + row < M) ? A[(int64_t)(m0 + row) * lda + k0 + kk] : 0.0f;
      Bs[kk][row] = (kin && n0 + row < N) ? B[(int64_t)(n0 + row) * ldb + k0 + kk] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void k_probe_f32(ProbeF32Args p) {
  const int m0 = blockIdx.y * ST, n0 = blockIdx.x * ST;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  simt_mainloop(p.X, p.ldx, p.T, m0, p.W, p.ldw, p.m, n0, p.n, acc);
  const int NC = p.r + p.R;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = m0 + ty * 4 + i;
    if (t >= p.T) continue;
    int kind = kKindForeground;
    if (p.has_side) kind = p.seq_kind[p.tok_seq[t]];
    float y4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int mm = n0 + tx * 4 + j;
      y4[j] = 0.0f;
      if (mm >= p.m) continue;
      float y = acc[i][j];
      if (kind >= kKindCentre) {   // foreground rows skip the side state entirely
        const float* ts = p.Tside + (int64_t)t * NC;
        float side = 0.0f;
        for (int jj = 0; jj < p.R; ++jj) side = fmaf(ts[p.r + jj], p.P[(int64_t)mm * p.R_cap + jj], side);
        if (kind >= 0) {
          const float* u = p.Uf + ((int64_t)kind * p.m + mm) * p.r;
          for (int jj = 0; jj < p.r; ++jj) side = fmaf(ts[jj], u[jj], side);
        }
        y += side;
      }
      if (p.bias) y += p.bias[mm];
      if (p.act == 1) y = fmaxf(y, 0.0f);
      y4[j] = y;
      if (p.act != 2) p.Y[(int64_t)t * p.ldy + mm] = y;
    }
    if (p.act == 2) {   // (gate, up) pairs of adjacent output features -> one output column each (m is even)
#pragma unroll
      for (int j = 0; j < 4; j += 2) {
        const int mm = n0 + tx * 4 + j;
        if (mm < p.m) p.Y[(int64_t)t * p.ldy + (mm >> 1)] = y4[j] / (1.0f + expf(-y4[j])) * y4[j + 1];
      }
    }
  }
}

hipError_t launch_probe_f32(const ProbeF32Args& a, hipStream_t st) {
  if (a.T == 0 || a.m == 0) return hipSuccess;
  if (a.has_side && a.r + a.R > 0) {
    const int64_t total = (int64_t)a.T * (a.r + a.R);
    hipLaunchKernelGGL(k_side_f32, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  }
  dim3 grid((a.m + ST - 1) / ST, (a.T + ST - 1) / ST);
  hipLaunchKernelGGL(k_probe_f32, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

int head_vocab_tiles_f32(int vocab) { return (vocab + ST - 1) / ST; }

// rows = tokens, columns = vocabulary; per (vocabulary tile, token): max logit,
// sum exp(z - max) and, where the target falls in the tile, the target logit.
__global__ __launch_bounds__(256) void k_head_f32(HeadScoreF32Args p) {
  const int m0 = blockIdx.y * ST, n0 = blockIdx.x * ST;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  simt_mainloop(p.H, p.ldh, p.T, m0, p.Wh, p.ldw, p.vocab, n0, p.d, acc);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = m0 + ty * 4 + i;
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (n0 + tx * 4 + j >= p.vocab) acc[i][j] = -INFINITY;
      mx = fmaxf(mx, acc[i][j]);
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) sum += expf(acc[i][j] - mx);
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o);
    if (t < p.T) {
      if (tx == 0) {
        p.part_max[(int64_t)blockIdx.x * p.T + t] = mx;
        p.part_sum[(int64_t)blockIdx.x * p.T + t] = sum;
      }
      const int loc = p.targets[t] - n0 - tx * 4;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (loc == j) p.tgt_logit[t] = acc[i][j];
    }
  }
}

hipError_t launch_head_score_f32(const HeadScoreF32Args& a, hipStream_t st) {
  if (a.T == 0) return hipSuccess;
  dim3 grid((a.vocab + ST - 1) / ST, (a.T + ST - 1) / ST);
  hipLaunchKernelGGL(k_head_f32, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace zo
