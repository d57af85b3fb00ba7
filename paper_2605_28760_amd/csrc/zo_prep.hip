// Preparation kernels: factor generation (Philox4x32-10 + Box-Muller; the
// seed-regenerated directions of Sec. 2.2 with the N(0,1) entries of Sec. 3.3),
// packing indices of the variable-length batch (Sec. 3.1) and the operand
// images the matrix-core kernels consume.
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

// ---- raw words / standalone factor fill ------------------------------------------
__global__ void k_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t first_block,
                               int64_t n_blocks, uint4* out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_blocks) return;
  out[i] = factor_block(seed, tensor_id, first_block + (uint64_t)i);
}

__global__ void k_factor_fill(uint64_t seed, uint32_t tensor_id, int64_t n_elems, int bf16, void* out) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q * 4 >= n_elems) return;
  const uint4 w = factor_block(seed, tensor_id, (uint64_t)q);
  float z[4];
  box_muller(w.x, w.y, z[0], z[1]);
  box_muller(w.z, w.w, z[2], z[3]);
#pragma unroll
  for (int l = 0; l < 4; ++l) {
    const int64_t e = q * 4 + l;
    if (e < n_elems) {
      if (bf16) ((bf16_t*)out)[e] = f32_to_bf16(z[l]);
      else ((float*)out)[e] = z[l];
    }
  }
}

hipError_t launch_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t first_block,
                               int64_t n_blocks, uint32_t* out, hipStream_t st) {
  if (n_blocks == 0) return hipSuccess;
  const int64_t grid = (n_blocks + 255) / 256;
  hipLaunchKernelGGL(k_philox_words, dim3((unsigned)grid), dim3(256), 0, st, seed, tensor_id, first_block,
                     n_blocks, (uint4*)out);
  return hipGetLastError();
}

hipError_t launch_factor_fill(uint64_t seed, uint32_t tensor_id, int64_t rows, int r, int bf16,
                              void* out, hipStream_t st) {
  const int64_t n = rows * r;
  if (n == 0) return hipSuccess;
  const int64_t blocks = (n + 3) / 4;
  hipLaunchKernelGGL(k_factor_fill, dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, st, seed,
                     tensor_id, n, bf16, out);
  return hipGetLastError();
}

// ---- packing indices -----------------------------------------------------------------
// tok_seq[t] = largest s with cu[s] <= t (empty sequences share an offset with
// their successor; the last of them is the one that owns row t).
__device__ __forceinline__ int seq_of_row(const int32_t* cu, int S, int t) {
  int lo = 0, hi = S;  // invariant: cu[lo] <= t, answer in [lo, hi)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ void tok_index_at(const BatchDev& b, int t, int32_t* tok_seq, int32_t* tok_cand) {
  if (t >= b.T) return;
  const int s = seq_of_row(b.cu, b.S, t);
  if (tok_seq) tok_seq[t] = s;
  if (tok_cand) tok_cand[t] = b.seq_cand[s];
}

__global__ void k_tok_index(BatchDev b, int32_t* tok_seq, int32_t* tok_cand) {
  tok_index_at(b, blockIdx.x * blockDim.x + threadIdx.x, tok_seq, tok_cand);
}

hipError_t launch_tok_index(const BatchDev& b, int32_t* tok_seq, int32_t* tok_cand, hipStream_t st) {
  if (b.T == 0) return hipSuccess;
  hipLaunchKernelGGL(k_tok_index, dim3((b.T + 255) / 256), dim3(256), 0, st, b, tok_seq, tok_cand);
  return hipGetLastError();
}

// Per-sequence kind / scale and the list of side-down work items (chunks of at
// most kSideRows rows of one sequence).  One workgroup; sequences are scanned in
// blocks of 1024 so the item order follows the row order.
__device__ __forceinline__ void seq_tables_block(const BatchDev& b, float eps, const SeqTables& t) {
  __shared__ int s_scan[1024];
  __shared__ int s_carry;
  const int tid = threadIdx.x;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < b.S; base += 1024) {
    const int s = base + tid;
    int row0 = 0, len = 0, kind = kKindForeground, nchunk = 0;
    float scale = 0.0f;
    if (s < b.S) {
      row0 = b.cu[s];
      len = max(b.cu[s + 1] - row0, 0);
      const int c = b.seq_cand[s];
      if (c >= 0 && c < b.C) {
        const int d = b.cand_dir[c];
        const float sg = b.cand_sign[c];
        if (d >= 0 && d < b.K && sg != 0.0f) { kind = d; scale = sg * eps; }
        else kind = kKindCentre;
      }
      t.seq_kind[s] = kind;
      t.seq_scale[s] = scale;
      nchunk = (len + kSideRows - 1) / kSideRows;
    }
    s_scan[tid] = nchunk;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const int v = (tid >= off) ? s_scan[tid - off] : 0;
      __syncthreads();
      s_scan[tid] += v;
      __syncthreads();
    }
    const int first = s_carry + s_scan[tid] - nchunk;
    for (int j = 0; j < nchunk; ++j) {
      if (first + j < t.max_items) {
        SideItem it;
        it.row0 = row0 + j * kSideRows;
        it.nrows = min(kSideRows, len - j * kSideRows);
        it.kind = kind;
        it.scale = scale;
        t.items[first + j] = it;
      }
    }
    __syncthreads();
    if (tid == 1023) s_carry += s_scan[1023];
    __syncthreads();
  }
  if (tid == 0) {
    const int n_items = min(s_carry, t.max_items);
    const int groups = max((n_items + 3) / 4, 1);
    t.n_items[0] = n_items;
    t.n_items[1] = max(1, min(t.side_ks_cap, t.side_slots / groups));
  }
}

__global__ __launch_bounds__(1024) void k_seq_tables(BatchDev b, float eps, SeqTables t) { seq_tables_block(b, eps, t); }

hipError_t launch_seq_tables(const BatchDev& b, float eps, const SeqTables& t, hipStream_t st) {
  hipLaunchKernelGGL(k_seq_tables, dim3(1), dim3(1024), 0, st, b, eps, t);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_tok_index(b, t.tok_seq, nullptr, st);
}

// ---- operand images ----------------------------------------------------------------------
// Four consecutive columns c0 .. c0+3 of row i of a [rows x r] factor: entries c >= r are zero.
// Entry (i, c) is element e = i*r + c of the stream, i.e. lane e%4 of block e/4; the four entries
// come out of one block when r is a multiple of 4 and out of two neighbouring blocks otherwise.
__device__ __forceinline__ void factor_quad(uint64_t seed, uint32_t tid, int64_t i, int r, int c0, float (&z)[4]) {
  const uint64_t e0 = (uint64_t)i * r + c0;
  float v[8];
  {
    const uint4 w = factor_block(seed, tid, e0 >> 2);
    box_muller(w.x, w.y, v[0], v[1]);
    box_muller(w.z, w.w, v[2], v[3]);
  }
  const int lane0 = (int)(e0 & 3);
  if (lane0 != 0) {
    const uint4 w = factor_block(seed, tid, (e0 >> 2) + 1);
    box_muller(w.x, w.y, v[4], v[5]);
    box_muller(w.z, w.w, v[6], v[7]);
  } else {
    v[4] = v[5] = v[6] = v[7] = 0.0f;
  }
#pragma unroll
  for (int l = 0; l < 4; ++l) {
    float x = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) x = (t == lane0 + l) ? v[t] : x;   // register select, no indexing
    z[l] = c0 + l < r ? x : 0.0f;
  }
}

// idx runs over [K][m][RP/4]: one thread writes four neighbouring entries of a row of U (8 bytes)
__device__ __forceinline__ void image_U_at(const BatchDev& b, int64_t idx, uint32_t tid_u, int m, int r, int RP, bf16_t* Uh) {
  const int quads = RP >> 2;
  const int64_t per_dir = (int64_t)m * quads;
  if (idx >= per_dir * b.K) return;
  const int k = (int)(idx / per_dir);
  const int64_t rem = idx - (int64_t)k * per_dir;
  const int i = (int)(rem / quads), c0 = (int)(rem % quads) * 4;
  float z[4] = {0.f, 0.f, 0.f, 0.f};
  if (c0 < r) factor_quad(b.seed[k], tid_u, i, r, c0, z);
  *reinterpret_cast<uint2*>(Uh + ((int64_t)k * m + i) * RP + c0) = make_uint2(pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3]));
}

// idx runs over [K][RP/4][n]: one thread writes entry i of four neighbouring rows of V^T
__device__ __forceinline__ void image_Vt_at(const BatchDev& b, int64_t idx, uint32_t tid_v, int n, int r, int RP, bf16_t* Vt) {
  const int quads = RP >> 2;
  const int64_t per_dir = (int64_t)n * quads;
  if (idx >= per_dir * b.K) return;
  const int k = (int)(idx / per_dir);
  const int64_t rem = idx - (int64_t)k * per_dir;
  const int c0 = (int)(rem / n) * 4, i = (int)(rem % n);
  float z[4] = {0.f, 0.f, 0.f, 0.f};
  if (c0 < r) factor_quad(b.seed_v ? b.seed_v[k] : b.seed[k], tid_v, i, r, c0, z);
#pragma unroll
  for (int l = 0; l < 4; ++l) Vt[((int64_t)k * RP + c0 + l) * n + i] = f32_to_bf16(z[l]);
}

__device__ __forceinline__ void image_P_at(int64_t idx, const float* P, int R_cap, int R_used, int Rp, int m, bf16_t* Ph) {
  if (idx >= (int64_t)m * Rp) return;
  const int i = (int)(idx / Rp), j = (int)(idx % Rp);
  Ph[idx] = f32_to_bf16(j < R_used ? P[(int64_t)i * R_cap + j] : 0.0f);
}

__global__ void k_factors_f32(BatchDev b, uint32_t tid, int rows, int r, float* out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_dir = (int64_t)rows * r;
  if (idx >= per_dir * b.K) return;
  const int k = (int)(idx / per_dir);
  const uint64_t seed = ((tid & 1u) && b.seed_v) ? b.seed_v[k] : b.seed[k];   // odd stream id: V
  out[idx] = factor_normal(seed, tid, (uint64_t)(idx - (int64_t)k * per_dir));
}

hipError_t launch_factors_f32(const BatchDev& b, uint32_t tensor_id, int m, int n, int r,
                              float* Uf, float* Vf, hipStream_t st) {
  if (b.K == 0) return hipSuccess;
  const int64_t nu = (int64_t)b.K * m * r, nv = (int64_t)b.K * n * r;
  hipLaunchKernelGGL(k_factors_f32, dim3((unsigned)((nu + 255) / 256)), dim3(256), 0, st, b, tensor_id & ~1u, m, r, Uf);
  hipLaunchKernelGGL(k_factors_f32, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, st, b, tensor_id | 1u, n, r, Vf);
  return hipGetLastError();
}

// ---- everything a bf16 probe linear prepares before its side-down pass, in one launch ------
// Block roles, in order: [sequence tables: 1] [token -> sequence map] [U image] [V^T image]
// [P image] [Vb^T image: 32x32 transposing tiles].  The pieces do not depend on one another.
struct ProbePrepArgs {
  BatchDev b; float eps; SeqTables tabs;
  uint32_t tensor_id; int m, n, r, RP, Rp;
  const float* P; const float* Vb; int R_cap, R_used;
  bf16_t* Uh; bf16_t* Vt; bf16_t* Ph; bf16_t* Vbt;
  int nb_tok, nb_U, nb_Vt, nb_P, nb_Vbt, vbt_tiles_n;
};

__global__ __launch_bounds__(1024) void k_probe_prep(ProbePrepArgs a) {
  int blk = blockIdx.x;
  if (blk == 0) { seq_tables_block(a.b, a.eps, a.tabs); return; }
  blk -= 1;
  if (blk < a.nb_tok) { tok_index_at(a.b, blk * 1024 + threadIdx.x, a.tabs.tok_seq, nullptr); return; }
  blk -= a.nb_tok;
  if (blk < a.nb_U) { image_U_at(a.b, (int64_t)blk * 1024 + threadIdx.x, a.tensor_id & ~1u, a.m, a.r, a.RP, a.Uh); return; }
  blk -= a.nb_U;
  if (blk < a.nb_Vt) { image_Vt_at(a.b, (int64_t)blk * 1024 + threadIdx.x, a.tensor_id | 1u, a.n, a.r, a.RP, a.Vt); return; }
  blk -= a.nb_Vt;
  if (blk < a.nb_P) { image_P_at((int64_t)blk * 1024 + threadIdx.x, a.P, a.R_cap, a.R_used, a.Rp, a.m, a.Ph); return; }
  blk -= a.nb_P;
  // Vbt[j][i] = Vb[i][j], one 32x32 tile per block, coalesced on both sides
  __shared__ float tile[32][33];
  const int i0 = (blk % a.vbt_tiles_n) * 32, j0 = (blk / a.vbt_tiles_n) * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  {
    const int i = i0 + ty, j = j0 + tx;
    tile[ty][tx] = (i < a.n && j < a.R_used) ? a.Vb[(int64_t)i * a.R_cap + j] : 0.0f;
  }
  __syncthreads();
  {
    const int j = j0 + ty, i = i0 + tx;
    if (j < a.Rp && i < a.n) a.Vbt[(int64_t)j * a.n + i] = f32_to_bf16(tile[tx][ty]);
  }
}

hipError_t launch_probe_prep_bf16(const BatchDev& b, float eps, const SeqTables& tabs, uint32_t tensor_id, int m,
                                  int n, int r, int RP, int Rp, const float* P, const float* Vb, int R_cap,
                                  int R_used, uint16_t* Uh, uint16_t* Vt, uint16_t* Ph, uint16_t* Vbt,
                                  hipStream_t st) {
  ProbePrepArgs a;
  a.b = b; a.eps = eps; a.tabs = tabs; a.tensor_id = tensor_id; a.m = m; a.n = n; a.r = r; a.RP = RP; a.Rp = Rp;
  a.P = P; a.Vb = Vb; a.R_cap = R_cap; a.R_used = R_used; a.Uh = Uh; a.Vt = Vt; a.Ph = Ph; a.Vbt = Vbt;
  auto blocks = [](int64_t n_elems) { return (int)((n_elems + 1023) / 1024); };
  a.nb_tok = blocks(b.T);
  a.nb_U = blocks((int64_t)b.K * m * (RP / 4));
  a.nb_Vt = blocks((int64_t)b.K * n * (RP / 4));
  a.nb_P = Rp > 0 ? blocks((int64_t)m * Rp) : 0;
  a.vbt_tiles_n = (n + 31) / 32;
  a.nb_Vbt = Rp > 0 ? a.vbt_tiles_n * ((Rp + 31) / 32) : 0;
  const int64_t total = 1 + (int64_t)a.nb_tok + a.nb_U + a.nb_Vt + a.nb_P + a.nb_Vbt;
  hipLaunchKernelGGL(k_probe_prep, dim3((unsigned)total), dim3(1024), 0, st, a);
  return hipGetLastError();
}

// ---- device-resident schedule of the multi-step loop (Sec. 3.2) ---------------------------
__global__ __launch_bounds__(256) void k_schedule_step(SchedDev* s, int nu, int n_blocks, int K, uint64_t base_u,
                                                       uint64_t base_v, uint64_t* seed_u, uint64_t* seed_v) {
  const int64_t t = s->next_step;
  __syncthreads();   // every thread has read the step number before thread 0 advances it
  const int64_t interval = t / nu;
  for (int j = threadIdx.x; j < K; j += blockDim.x) {
    seed_u[j] = base_u + (uint64_t)t * (uint64_t)K + (uint64_t)j;
    seed_v[j] = base_v + (uint64_t)interval * (uint64_t)K + (uint64_t)j;
  }
  if (threadIdx.x == 0) {
    s->step = t;
    s->interval = (int32_t)interval;
    s->block = (int32_t)(interval % n_blocks);
    s->append = (t % nu == 0) ? 1 : 0;
    s->reserved = 0;
    s->next_step = t + 1;
  }
}

hipError_t launch_schedule_step(SchedDev* s, int nu, int n_blocks, int K, uint64_t base_u, uint64_t base_v,
                                uint64_t* seed_u, uint64_t* seed_v, hipStream_t st) {
  hipLaunchKernelGGL(k_schedule_step, dim3(1), dim3(256), 0, st, s, nu, n_blocks, K, base_u, base_v, seed_u, seed_v);
  return hipGetLastError();
}

}  // namespace zo
