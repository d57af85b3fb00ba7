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

// Exclusive prefix sum of one value per thread over a block of 1024 threads; *total = the block's sum.
__device__ __forceinline__ int block_scan_1024(int v, int* s_scan, int* total) {
  const int tid = threadIdx.x;
  s_scan[tid] = v;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int u = (tid >= off) ? s_scan[tid - off] : 0;
    __syncthreads();
    s_scan[tid] += u;
    __syncthreads();
  }
  const int incl = s_scan[tid];
  *total = s_scan[1023];
  __syncthreads();
  return incl - v;
}

// Per-sequence kind / scale, the list of side-down work items (chunks of at
// most item_rows rows of one sequence) and, for the bf16 GEMM, the side K tiles of
// every token tile.  One workgroup; sequences and tiles are scanned in blocks of
// 1024 so the item order follows the row order.
__device__ __forceinline__ void seq_tables_block(const BatchDev& b, float eps, const SeqTables& t) {
  __shared__ int s_scan[1024];
  const int tid = threadIdx.x;
  int carry = 0;
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
      // (a foreground sequence has no side term: no items, none of its rows is read by the side-down pass)
      nchunk = kind == kKindForeground ? 0 : (len + t.item_rows - 1) / t.item_rows;
    }
    int total;
    const int first = carry + block_scan_1024(nchunk, s_scan, &total);
    for (int j = 0; j < nchunk; ++j) {
      if (first + j < t.max_items) {
        SideItem it;
        it.row0 = row0 + j * t.item_rows;
        it.nrows = min(t.item_rows, len - j * t.item_rows);
        it.kind = kind;
        it.scale = scale;
        t.items[first + j] = it;
      }
    }
    carry += total;
  }
  if (tid == 0) t.n_items[0] = min(carry, t.max_items);
  if (!t.tile_hdr) return;

  // Token tiles.  A tile's slot list names the distinct directions of the sequences that intersect it, in
  // order of first appearance, SPD slots each; it lives in a region of the list sized by the number of
  // those sequences (the sum over the tiles is at most the tiles plus the sequences).  Kinds written by
  // other threads of this workgroup above are visible after the barriers of the scans.
  __syncthreads();
  int slot_carry = 0, kt_carry = 0;
  for (int base = 0; base < t.n_tn; base += 1024) {
    const int tn = base + tid;
    int t0 = 0, t1 = 0, s_first = 0, s_last = -1, bound = 0;
    if (tn < t.n_tn) {
      t0 = tn * kTileN;
      t1 = min(b.T, t0 + kTileN);
      s_first = seq_of_row(b.cu, b.S, t0);
      s_last = seq_of_row(b.cu, b.S, t1 - 1);
      bound = min(min(s_last - s_first + 1, b.K), kTileN) * t.SPD;   // a tile meets at most kTileN non-empty sequences
    }
    int total;
    const int slot0 = slot_carry + block_scan_1024(bound, s_scan, &total);
    slot_carry += total;
    int q = 0, n_kt = 0, n_bank = 0;
    if (tn < t.n_tn) {
      bool any = false;
      for (int s = s_first; s <= s_last; ++s) {
        if (min(b.cu[s + 1], t1) <= max(b.cu[s], t0)) continue;   // no row of s in this tile
        const int kind = t.seq_kind[s];
        if (kind >= kKindCentre) any = true;
        if (kind < 0) continue;
        bool seen = false;
        for (int j = 0; j < q && !seen; ++j) seen = t.tile_slots[slot0 + j * t.SPD] == kind * t.SPD;
        if (!seen && slot0 + (q + 1) * t.SPD <= t.slot_cap) {
          for (int blk = 0; blk < t.SPD; ++blk) t.tile_slots[slot0 + q * t.SPD + blk] = kind * t.SPD + blk;
          ++q;
        }
      }
      n_bank = any ? t.RpT : 0;
      n_kt = (q * t.SPD + 1) / 2 + n_bank;
    }
    const int kt0 = kt_carry + block_scan_1024(n_kt, s_scan, &total);
    kt_carry += total;
    if (tn < t.n_tn) {
      TileHdr h;
      h.kt0 = kt0; h.n_slots = q * t.SPD; h.n_bank_kt = n_bank; h.slot0 = slot0;
      if (kt0 + n_kt > t.kt_cap) { h.n_slots = 0; h.n_bank_kt = 0; n_kt = 0; }   // cannot happen: the caps are bounds
      t.tile_hdr[tn] = h;
      for (int j = 0; j < n_kt; ++j) t.kt_tile[kt0 + j] = tn;
    }
  }
  if (tid == 0) t.n_items[1] = min(kt_carry, t.kt_cap);
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

// idx = (a * per_a) + b * inner + c with b * inner + c < per_a and c < inner.  32-bit divisions when the numbers
// allow (a 64-bit division costs more instructions than the normals a thread generates).
__device__ __forceinline__ void split3(int64_t idx, int64_t per_a, int inner, int& a, int& b, int& c) {
  if (idx < (1ll << 31) && per_a < (1ll << 31)) {
    const uint32_t x = (uint32_t)idx, pa = (uint32_t)per_a;
    const uint32_t qa = x / pa, rem = x - qa * pa;
    const uint32_t qb = rem / (uint32_t)inner;
    a = (int)qa; b = (int)qb; c = (int)(rem - qb * (uint32_t)inner);
  } else {
    const int64_t qa = idx / per_a, rem = idx - qa * per_a;
    const int64_t qb = rem / inner;
    a = (int)qa; b = (int)qb; c = (int)(rem - qb * inner);
  }
}

// idx runs over [K][m_img][RP32/4]: one thread writes four neighbouring entries of a row of U (8 bytes) into
// the image [K * SPD][m_img][32]; rows >= m and columns >= r are zero
__device__ __forceinline__ void image_U_at(const BatchDev& b, int64_t idx, uint32_t tid_u, int m, int m_img, int r, int SPD,
                                           bf16_t* Uimg) {
  const int quads = SPD * 8;
  const int64_t per_dir = (int64_t)m_img * quads;
  if (idx >= per_dir * b.K) return;
  int k, i, c0;
  split3(idx, per_dir, quads, k, i, c0);
  c0 *= 4;
  float z[4] = {0.f, 0.f, 0.f, 0.f};
  if (i < m && c0 < r) factor_quad(b.seed[k], tid_u, i, r, c0, z);
  *reinterpret_cast<uint2*>(Uimg + (((int64_t)k * SPD + (c0 >> 5)) * m_img + i) * 32 + (c0 & 31)) =
      make_uint2(pack_bf16x2(z[0], z[1]), pack_bf16x2(z[2], z[3]));
}

// idx runs over [K][RP/4][n]: one thread writes entry i of four neighbouring rows of V^T
__device__ __forceinline__ void image_Vt_at(const BatchDev& b, int64_t idx, uint32_t tid_v, int n, int r, int RP, bf16_t* Vt) {
  const int quads = RP >> 2;
  const int64_t per_dir = (int64_t)n * quads;
  if (idx >= per_dir * b.K) return;
  int k, c0, i;
  split3(idx, per_dir, n, k, c0, i);
  c0 *= 4;
  float z[4] = {0.f, 0.f, 0.f, 0.f};
  if (c0 < r) factor_quad(b.seed_v ? b.seed_v[k] : b.seed[k], tid_v, i, r, c0, z);
#pragma unroll
  for (int l = 0; l < 4; ++l) Vt[((int64_t)k * RP + c0 + l) * n + i] = f32_to_bf16(z[l]);
}

// idx runs over [m_img][RpT * 64]: image [RpT][m_img][64] of P; rows >= m and columns >= R_used are zero
__device__ __forceinline__ void image_P_at(int64_t idx, const float* P, int R_cap, int R_used, int RpT, int m, int m_img,
                                           bf16_t* Pimg) {
  const int cols = RpT * 64;
  if (idx >= (int64_t)m_img * cols) return;
  int zero, i, j;
  split3(idx, (int64_t)m_img * cols, cols, zero, i, j);
  Pimg[((int64_t)(j >> 6) * m_img + i) * 64 + (j & 63)] = f32_to_bf16(i < m && j < R_used ? P[(int64_t)i * R_cap + j] : 0.0f);
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
  uint32_t tensor_id; int m, n, r, RP, Rp, m_img;
  const float* P; const float* Vb; int R_cap, R_used;
  bf16_t* Uimg; bf16_t* Vt; bf16_t* Pimg; bf16_t* Vbt;
  int nb_tok, nb_U, nb_Vt, nb_P, nb_Vbt, vbt_tiles_n;
};

__global__ __launch_bounds__(1024) void k_probe_prep(ProbePrepArgs a) {
  int blk = blockIdx.x;
  if (blk == 0) { seq_tables_block(a.b, a.eps, a.tabs); return; }
  blk -= 1;
  if (blk < a.nb_tok) { tok_index_at(a.b, blk * 1024 + threadIdx.x, a.tabs.tok_seq, nullptr); return; }
  blk -= a.nb_tok;
  if (blk < a.nb_U) { image_U_at(a.b, (int64_t)blk * 1024 + threadIdx.x, a.tensor_id & ~1u, a.m, a.m_img, a.r, a.tabs.SPD, a.Uimg); return; }
  blk -= a.nb_U;
  if (blk < a.nb_Vt) { image_Vt_at(a.b, (int64_t)blk * 1024 + threadIdx.x, a.tensor_id | 1u, a.n, a.r, a.RP, a.Vt); return; }
  blk -= a.nb_Vt;
  if (blk < a.nb_P) { image_P_at((int64_t)blk * 1024 + threadIdx.x, a.P, a.R_cap, a.R_used, a.tabs.RpT, a.m, a.m_img, a.Pimg); return; }
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
                                  int R_used, int m_img, uint16_t* Uimg, uint16_t* Vt, uint16_t* Pimg, uint16_t* Vbt,
                                  hipStream_t st) {
  ProbePrepArgs a;
  a.b = b; a.eps = eps; a.tabs = tabs; a.tensor_id = tensor_id; a.m = m; a.n = n; a.r = r; a.RP = RP; a.Rp = Rp;
  a.P = P; a.Vb = Vb; a.R_cap = R_cap; a.R_used = R_used; a.Uimg = Uimg; a.Vt = Vt; a.Pimg = Pimg; a.Vbt = Vbt;
  a.m_img = m_img;
  auto blocks = [](int64_t n_elems) { return (int)((n_elems + 1023) / 1024); };
  a.nb_tok = blocks(b.T);
  a.nb_U = blocks((int64_t)b.K * m_img * (tabs.SPD * 8));
  a.nb_Vt = blocks((int64_t)b.K * n * (RP / 4));
  a.nb_P = Rp > 0 ? blocks((int64_t)m_img * tabs.RpT * 64) : 0;
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
