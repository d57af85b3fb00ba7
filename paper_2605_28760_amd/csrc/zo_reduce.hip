// Small reduction kernels: merging the per-vocabulary-tile softmax partials
// into token / sequence / candidate NLL (Sec. 3.3: device-resident per-request
// NLL), the antithetic two-point estimate (Sec. 2.1, Eq. 2) and the lazy bank
// update (Sec. 3.2, Eq. "layer-coupling").  All reductions run in a fixed
// order; a sequence's sum is ordered relative to its own first row, so it does
// not depend on where the sequence sits in the packed batch.
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

// 32 tokens per workgroup, 8 threads per token: thread j of a token folds vocabulary
// tiles j, j+8, ... (coalesced over tokens), then the 8 partial (max, sum) pairs are
// merged in a fixed order.
__global__ __launch_bounds__(256) void k_tok_nll(ScoreCombineArgs a) {
  __shared__ float s_m[8][33], s_s[8][33];
  const int tl = threadIdx.x & 31, j0 = threadIdx.x >> 5;
  const int t = blockIdx.x * 32 + tl;
  float M = -INFINITY, S = 0.0f;
  const int at = (t < a.T && a.pos) ? a.pos[t] : t;   // where this token's partials are
  if (t < a.T && a.targets[t] >= 0) {
    // four tiles per trip so that their loads are in flight together; merged in the same order as one by one
    for (int j = j0; j < a.n_vt; j += 32) {
      float m[4], s[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int jj = j + 8 * u;
        const bool in = jj < a.n_vt;
        m[u] = in ? a.part_max[(int64_t)jj * a.T + at] : -INFINITY;
        s[u] = in ? a.part_sum[(int64_t)jj * a.T + at] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j + 8 * u >= a.n_vt) break;
        const float Mn = fmaxf(M, m[u]);
        if (Mn > -INFINITY) S = S * expf(M - Mn) + s[u] * expf(m[u] - Mn);
        M = Mn;
      }
    }
  }
  s_m[j0][tl] = M;
  s_s[j0][tl] = S;
  __syncthreads();
  if (j0 == 0 && t < a.T) {
    if (a.targets[t] < 0) { a.tok_nll[t] = 0.0f; return; }
    float Mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) Mx = fmaxf(Mx, s_m[j][tl]);
    float Sx = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s_m[j][tl] > -INFINITY) Sx += s_s[j][tl] * expf(s_m[j][tl] - Mx);
    a.tok_nll[t] = (Mx + logf(Sx)) - a.tgt_logit[at];
  }
}

// One workgroup per sequence: thread i takes rows i, i+256, ... of the sequence,
// then a fixed binary tree over the 256 partial sums.
__global__ __launch_bounds__(256) void k_seq_nll(ScoreCombineArgs a) {
  __shared__ float s_sum[256];
  __shared__ int s_cnt[256];
  const int s = blockIdx.x, tid = threadIdx.x;
  const int lo = a.cu[s], hi = a.cu[s + 1];
  float sum = 0.0f;
  int cnt = 0;
  for (int t = lo + tid; t < hi; t += 256) {
    sum += a.tok_nll[t];
    cnt += a.targets[t] >= 0 ? 1 : 0;
  }
  s_sum[tid] = sum;
  s_cnt[tid] = cnt;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (tid < off) { s_sum[tid] += s_sum[tid + off]; s_cnt[tid] += s_cnt[tid + off]; }
    __syncthreads();
  }
  if (tid == 0) { a.seq_nll[s] = s_sum[0]; a.seq_cnt[s] = s_cnt[0]; }
}

// One wave per candidate.  The candidate's sequences are folded strictly in sequence
// order (64 candidates-id loads at a time, then the matching ones one by one), so the sum
// depends only on the ordered list of that candidate's own sequences, not on what else
// is in the batch.
__global__ __launch_bounds__(64) void k_cand_sum(ScoreCombineArgs a) {
  const int c = blockIdx.x, lane = threadIdx.x;
  float sum = 0.0f;
  int cnt = 0;
  for (int base = 0; base < a.S; base += 64) {
    const int s = base + lane;
    const bool match = s < a.S && a.seq_cand[s] == c;
    const float v = match ? a.seq_nll[s] : 0.0f;
    const int n = match ? a.seq_cnt[s] : 0;
    uint64_t mask = __ballot(match);
    while (mask) {
      const int b = __ffsll((unsigned long long)mask) - 1;
      sum += __shfl(v, b);
      cnt += __shfl(n, b);
      mask &= mask - 1;
    }
  }
  if (lane == 0) { a.cand_sum[c] = sum; a.cand_cnt[c] = cnt; }
}

// The scored tokens (Sec. 3.3: only active tokens need logits), in ascending order.  One
// workgroup of 16 waves; wave w owns a contiguous range of tokens and walks it 64 at a time
// (coalesced reads, ballot + popcount), first counting, then, after a scan over the 16 wave
// totals, writing the list and every token's position in it.
__global__ __launch_bounds__(1024) void k_active_rows(const int32_t* targets, int T, int32_t* rows, int32_t* pos,
                                                      int32_t* n_rows) {
  __shared__ int s_tot[16];
  constexpr int U = 16;  // 64-token pieces loaded together (independent loads: one round trip per 1024 tokens)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int per_wave = ((T + 15) / 16 + 63) / 64 * 64;
  const int lo = min(wave * per_wave, T), hi = min(lo + per_wave, T);
  int cnt = 0;
  for (int t0 = lo; t0 < hi; t0 += 64 * U) {
    int32_t tg[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) tg[u] = targets[min(t0 + u * 64 + lane, T - 1)];   // unconditional: the loads go out together
#pragma unroll
    for (int u = 0; u < U; ++u) on[u] = t0 + u * 64 + lane < hi && tg[u] >= 0;
#pragma unroll
    for (int u = 0; u < U; ++u) cnt += __popcll(__ballot(on[u]));
  }
  if (lane == 0) s_tot[wave] = cnt;
  __syncthreads();
  int base = 0, total = 0;
  for (int w = 0; w < 16; ++w) {
    if (w < wave) base += s_tot[w];
    total += s_tot[w];
  }
  for (int t0 = lo; t0 < hi; t0 += 64 * U) {
    int32_t tg[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) tg[u] = targets[min(t0 + u * 64 + lane, T - 1)];   // unconditional: the loads go out together
#pragma unroll
    for (int u = 0; u < U; ++u) on[u] = t0 + u * 64 + lane < hi && tg[u] >= 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * 64 + lane;
      const uint64_t m = __ballot(on[u]);
      const int before = __popcll(m & ((1ull << lane) - 1ull));
      if (t < hi) pos[t] = base + before;
      if (on[u]) rows[base + before] = t;
      base += __popcll(m);
    }
  }
  if (threadIdx.x == 0) *n_rows = total;
}

hipError_t launch_active_rows(const int32_t* targets, int T, int32_t* rows, int32_t* pos, int32_t* n_rows,
                              hipStream_t st) {
  hipLaunchKernelGGL(k_active_rows, dim3(1), dim3(1024), 0, st, targets, T, rows, pos, n_rows);
  return hipGetLastError();
}

hipError_t launch_score_combine(const ScoreCombineArgs& a, hipStream_t st) {
  if (a.T > 0) hipLaunchKernelGGL(k_tok_nll, dim3((a.T + 31) / 32), dim3(256), 0, st, a);
  if (a.S > 0) hipLaunchKernelGGL(k_seq_nll, dim3(a.S), dim3(256), 0, st, a);
  if (a.C > 0) hipLaunchKernelGGL(k_cand_sum, dim3(a.C), dim3(64), 0, st, a);
  return hipGetLastError();
}

__global__ void k_estimate(BatchDev b, const float* cand_sum, const int32_t* cand_cnt, float eps,
                           int reduction, float* cand_loss, float* proj_grad) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  auto loss_of = [&](int c) {
    return reduction == 0 ? cand_sum[c] / (float)max(cand_cnt[c], 1) : cand_sum[c];
  };
  if (i < b.C) cand_loss[i] = loss_of(i);
  if (i < b.K) {
    int cp = -1, cm = -1;
    for (int c = 0; c < b.C; ++c) {
      if (b.cand_dir[c] != i) continue;
      const float sg = b.cand_sign[c];
      if (sg > 0.0f && cp < 0) cp = c;
      if (sg < 0.0f && cm < 0) cm = c;
    }
    proj_grad[i] = (cp >= 0 && cm >= 0) ? (loss_of(cp) - loss_of(cm)) / (2.0f * eps) : 0.0f;
  }
}

hipError_t launch_estimate(const BatchDev& b, const float* cand_sum, const int32_t* cand_cnt, float eps,
                           int reduction, float* cand_loss, float* proj_grad, hipStream_t st) {
  const int n = b.C > b.K ? b.C : b.K;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_estimate, dim3((n + 63) / 64), dim3(64), 0, st, b, cand_sum, cand_cnt, eps, reduction,
                     cand_loss, proj_grad);
  return hipGetLastError();
}

// Reward-normalised one-sided estimate: one workgroup; every direction finds its representative
// candidate, thread 0 forms mean and variance of the rewards in direction order (fixed order, N is
// small), then every direction gets -z / eps.
__global__ __launch_bounds__(256) void k_estimate_es(BatchDev b, const float* cand_sum, const int32_t* cand_cnt,
                                                     float eps, int reduction, float* cand_loss, float* proj_grad) {
  __shared__ float s_mean, s_inv_std;
  auto loss_of = [&](int c) {
    return reduction == 0 ? cand_sum[c] / (float)max(cand_cnt[c], 1) : cand_sum[c];
  };
  auto rep_of = [&](int k) {
    for (int c = 0; c < b.C; ++c)
      if (b.cand_dir[c] == k && b.cand_sign[c] > 0.0f) return c;
    return -1;
  };
  for (int c = threadIdx.x; c < b.C; c += blockDim.x) cand_loss[c] = loss_of(c);
  if (threadIdx.x == 0) {
    float sum = 0.0f;
    int n = 0;
    for (int k = 0; k < b.K; ++k) {
      const int c = rep_of(k);
      if (c >= 0) { sum += -loss_of(c); ++n; }
    }
    const float mean = n > 0 ? sum / (float)n : 0.0f;
    float var = 0.0f;
    for (int k = 0; k < b.K; ++k) {
      const int c = rep_of(k);
      if (c >= 0) { const float dlt = -loss_of(c) - mean; var = fmaf(dlt, dlt, var); }
    }
    var = n > 0 ? var / (float)n : 0.0f;
    s_mean = mean;
    s_inv_std = 1.0f / fmaxf(sqrtf(var), 1e-8f);
  }
  __syncthreads();
  for (int k = threadIdx.x; k < b.K; k += blockDim.x) {
    const int c = rep_of(k);
    proj_grad[k] = c >= 0 ? -((-loss_of(c) - s_mean) * s_inv_std) / eps : 0.0f;
  }
}

hipError_t launch_estimate_es(const BatchDev& b, const float* cand_sum, const int32_t* cand_cnt, float eps,
                              int reduction, float* cand_loss, float* proj_grad, hipStream_t st) {
  if (b.C == 0 && b.K == 0) return hipSuccess;
  hipLaunchKernelGGL(k_estimate_es, dim3(1), dim3(256), 0, st, b, cand_sum, cand_cnt, eps, reduction, cand_loss,
                     proj_grad);
  return hipGetLastError();
}

// ---- lazy bank update ---------------------------------------------------------------------
constexpr int kBankBatch = 32;
struct BankCols { int32_t first_dir; int32_t n; int32_t col0[kBankBatch]; };

// Four consecutive entries 4q .. 4q+3 of a [rows x r] factor stream scaled into `dst` (a row-major matrix
// of pitch R_cap, the factor's block starting at column col0): dst = beta * f (set) or dst += beta * f.
// One Philox block yields the four normals.  When the rank is a multiple of 4 the four entries are
// neighbours in one row, and if the block is 16-byte aligned they move as one float4.
template <bool kAccumulate>
__device__ __forceinline__ void bank_quad(float* M, int R_cap, int col0, int rows, int r, uint64_t seed, uint32_t tid,
                                          int64_t q, float beta, bool bf16) {
  const int64_t e0 = q * 4, total = (int64_t)rows * r;
  if (e0 >= total) return;
  const uint4 w = factor_block(seed, tid, (uint64_t)q);
  float z[4];
  box_muller(w.x, w.y, z[0], z[1]);
  box_muller(w.z, w.w, z[2], z[3]);
#pragma unroll
  for (int l = 0; l < 4; ++l) {
    if (bf16) z[l] = bf16_round(z[l]);
    z[l] *= beta;
  }
  // (32-bit division when the factor has fewer than 2^31 entries: the 64-bit one costs more than the normals)
  const int i = total < (1ll << 31) ? (int)((uint32_t)e0 / (uint32_t)r) : (int)(e0 / r);
  const int j = (int)(e0 - (int64_t)i * r);
  float* dst = M + (int64_t)i * R_cap + col0 + j;
  if ((r & 3) == 0 && (((uintptr_t)dst) & 15u) == 0) {
    float4 v = make_float4(z[0], z[1], z[2], z[3]);
    if (kAccumulate) {
      const float4 old = *reinterpret_cast<const float4*>(dst);
      v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
    }
    *reinterpret_cast<float4*>(dst) = v;
    return;
  }
#pragma unroll
  for (int l = 0; l < 4; ++l) {
    const int64_t e = e0 + l;
    if (e >= total) break;
    float* d1 = M + (e / r) * R_cap + col0 + (int)(e % r);
    *d1 = kAccumulate ? *d1 + z[l] : z[l];
  }
}

// Quad q of direction kb (within the batch `cols`) of one layer's update.
__device__ __forceinline__ void bank_update_entry(const BankUpdateArgs& a, const BankCols& cols, int kb, int64_t q) {
  const int k = cols.first_dir + kb;
  // block and mode: from the host (by value) or from the device-resident schedule
  const int col0 = a.sched ? (a.sched->block * a.n_dirs + k) * a.r : cols.col0[kb];
  const bool append = a.sched ? a.sched->append != 0 : a.append != 0;
  if (col0 < 0 || col0 + a.r > a.R_cap) return;
  const float w = a.dir_weight ? a.dir_weight[k] : a.default_weight;
  const float beta = -a.lr * a.proj_grad[k] * w;
  if (append) {
    bank_quad<false>(a.P, a.R_cap, col0, a.m, a.r, a.seed[k], a.tensor_id & ~1u, q, beta, a.bf16);
    bank_quad<false>(a.Vb, a.R_cap, col0, a.n, a.r, a.seed_v ? a.seed_v[k] : a.seed[k], a.tensor_id | 1u, q, 1.0f, a.bf16);
  } else {
    bank_quad<true>(a.P, a.R_cap, col0, a.m, a.r, a.seed[k], a.tensor_id & ~1u, q, beta, a.bf16);
  }
}

// grid.y = direction within the batch; grid.x covers the quads of max(m, n) * r entries.
__global__ void k_bank_update(BankUpdateArgs a, BankCols cols) {
  bank_update_entry(a, cols, blockIdx.y, (int64_t)blockIdx.x * blockDim.x + threadIdx.x);
}

// The same update for many layers in one launch (grid.z = layer): at the paper's sizes one layer's
// update is a few hundred KB and its launch costs more than its traffic.
__global__ void k_bank_update_multi(BankUpdateArgs a, BankCols cols, BankLayerSet layers) {
  const BankLayer& l = layers.l[blockIdx.z];
  a.P = l.P; a.Vb = l.Vb; a.R_cap = l.R_cap; a.m = l.m; a.n = l.n; a.tensor_id = l.tensor_id;
  bank_update_entry(a, cols, blockIdx.y, (int64_t)blockIdx.x * blockDim.x + threadIdx.x);
}

hipError_t launch_bank_update(const BankUpdateArgs& a, int n_dirs, const int32_t* col0, hipStream_t st) {
  const int rows = (a.append || a.sched) ? (a.m > a.n ? a.m : a.n) : a.m;
  const int64_t total = ((int64_t)rows * a.r + 3) / 4;   // quads: a thread takes four entries
  if (total == 0) return hipSuccess;
  for (int first = 0; first < n_dirs; first += kBankBatch) {
    BankCols cols;
    cols.first_dir = first;
    cols.n = n_dirs - first < kBankBatch ? n_dirs - first : kBankBatch;
    for (int i = 0; i < kBankBatch; ++i) cols.col0[i] = (col0 && i < cols.n) ? col0[first + i] : 0;
    hipLaunchKernelGGL(k_bank_update, dim3((unsigned)((total + 255) / 256), cols.n), dim3(256), 0, st, a, cols);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_bank_update_multi(const BankUpdateArgs& common, const BankLayer* layers, int n_layers, int n_dirs,
                                    const int32_t* col0, hipStream_t st) {
  for (int l0 = 0; l0 < n_layers; l0 += kBankMaxLayers) {
    BankLayerSet set;
    const int nl = n_layers - l0 < kBankMaxLayers ? n_layers - l0 : kBankMaxLayers;
    int64_t total = 0;
    for (int i = 0; i < kBankMaxLayers; ++i) {
      set.l[i] = layers[l0 + (i < nl ? i : 0)];
      const BankLayer& l = set.l[i];
      const int rows = common.append ? (l.m > l.n ? l.m : l.n) : l.m;
      if (i < nl && ((int64_t)rows * common.r + 3) / 4 > total) total = ((int64_t)rows * common.r + 3) / 4;
    }
    if (total == 0) continue;
    for (int first = 0; first < n_dirs; first += kBankBatch) {
      BankCols cols;
      cols.first_dir = first;
      cols.n = n_dirs - first < kBankBatch ? n_dirs - first : kBankBatch;
      for (int i = 0; i < kBankBatch; ++i) cols.col0[i] = i < cols.n ? col0[first + i] : 0;
      hipLaunchKernelGGL(k_bank_update_multi, dim3((unsigned)((total + 255) / 256), cols.n, nl), dim3(256), 0, st, common,
                         cols, set);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace zo
