// Matrix-core kernels for gfx950: the probe linear (Sec. 3.2: every candidate
// row sees W_0 + s eps U V^T + P Vb^T, applied as factors) and the fused
// LM-head scoring (Sec. 3.3: per-request NLL without materialising logits).
//
// Both are one 256x256x64-tiled bf16 GEMM with fp32 accumulation on
// v_mfma_f32_32x32x16_bf16.  Four waves in a 2x2 grid own 128x128 each.  Tiles
// of both operands stream global -> LDS with direct-to-LDS loads into a
// double-buffered, XOR-swizzled layout; workgroups are rasterised so that the
// 32 workgroups resident on one XCD share an 8x4 block of output tiles.
//
// Determinism / batch invariance: the tile shape and the K order never depend
// on the batch, there is no split-K and no atomic, so a row's result depends
// only on that row's operands.
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

constexpr int BM = kTileM, BN = kTileN, BK = kTileK;
constexpr int kOperandStage = BM * BK * 2;        // 32 KiB: one operand tile (256 rows x 128 B)
constexpr int kStage = 2 * kOperandStage;         // A tile then B tile
constexpr int kGemmLds = 2 * kStage;              // double buffered: 128 KiB
constexpr int kGroupM = 8;                        // raster: tile rows per group
constexpr int kXcds = 8;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// blockIdx -> output tile.  Hardware deals consecutive workgroup ids round-robin
// to the 8 XCDs; id = xcd + 8 * local.  Each XCD gets a contiguous range of the
// grouped raster, so the workgroups that share an L2 work on neighbouring tiles.
__device__ __forceinline__ bool tile_of_block(int bid, int n_tm, int n_tn, int& tm, int& tn) {
  const int total = n_tm * n_tn;
  const int per_xcd = (total + kXcds - 1) / kXcds;
  const int L = (bid % kXcds) * per_xcd + bid / kXcds;
  if (L >= total) return false;
  const int per_group = kGroupM * n_tn;
  const int g = L / per_group, in_g = L - g * per_group;
  const int first_m = g * kGroupM;
  const int gsize = min(n_tm - first_m, kGroupM);
  tm = first_m + in_g % gsize;
  tn = in_g / gsize;
  return true;
}

__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Main loop: acc[rb][cb] += A[tile rows] * B[tile rows]^T over K (multiple of 64).
// A and B are row-major with K contiguous; rows beyond M / N are clamped to the
// last valid row (their results are never stored).
//
// Pipeline.  K tiles of 64 (128-byte row segments, so every L2 request is a full
// line) alternate between two LDS stages.  A tile is four k-steps of 16; MFMA
// fragments are double buffered in registers and the LDS reads of the next
// k-step run under the 16 MFMAs of the current one.  The 16 direct-to-LDS loads
// a wave issues per tile are spread thinly (one per ~3 MFMAs) over k-step 3 of
// the previous tile and k-steps 0..1 of the current one: a burst would fill the
// memory pipeline's queues and stall the wave, and with it the MFMA stream.
// The single barrier of a tile sits before k-step 3: by then every wave has
// read its last fragments of this tile's stage (so the stage can be refilled)
// and the next tile has landed (so its first fragments can be fetched under
// k-step 3).
__device__ __forceinline__ void gemm_mainloop(const bf16_t* __restrict__ A, int64_t lda, int M, int tile_m0,
                                              const bf16_t* __restrict__ B, int64_t ldb, int N, int tile_n0,
                                              int K, f32x16 (&acc)[4][4], char* lds) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;

  // global -> LDS mapping: load j (0..7) of this wave fills the 1 KiB block (wave*8 + j)
  // of an operand tile: 8 rows x 128 B.  Lane i lands at byte 16*i of the block, i.e. row
  // i/8, physical chunk i%8, which holds logical chunk (i%8) ^ ((row>>1)&7).
  uint32_t offA[8], offB[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = (wave * 8 + j) * 8 + (lane >> 3);
    const int lch = (lane & 7) ^ ((row >> 1) & 7);
    const int ra = min(tile_m0 + row, M - 1) - tile_m0;
    const int rbn = min(tile_n0 + row, N - 1) - tile_n0;
    offA[j] = (uint32_t)((int64_t)ra * lda * 2 + lch * 16);
    offB[j] = (uint32_t)((int64_t)rbn * ldb * 2 + lch * 16);
  }
  // Buffer resources over the rows of this tile: one 32-bit per-lane offset and a scalar
  // K offset per load, no 64-bit address arithmetic in the loop.  Reads past the end of
  // the matrix (none are issued: rows are clamped) would return zero instead of faulting.
  const int64_t bytesA = ((int64_t)(M - tile_m0 - 1) * lda + K) * 2;
  const int64_t bytesB = ((int64_t)(N - tile_n0 - 1) * ldb + K) * 2;
  const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(A + (int64_t)tile_m0 * lda), 0, (int)min(bytesA, (int64_t)0x7FFFFFFF), 0x00020000);
  const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(B + (int64_t)tile_n0 * ldb), 0, (int)min(bytesB, (int64_t)0x7FFFFFFF), 0x00020000);

  // LDS -> register mapping (32x32x16 fragments: lane l holds row l%32, k-group l/32)
  const int lrow = lane & 31;
  const int swz = (lrow >> 1) & 7;
  uint32_t roff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) roff[kk] = lrow * 128 + (((kk * 2 + (lane >> 5)) ^ swz) << 4);
  const uint32_t aBase = wm * 128 * 128, bBase = kOperandStage + wn * 128 * 128;

  // load i (0..15) of tile kt: i < 8 -> A chunk i, else B chunk i - 8
  auto issue_range = [&](int stage, int kt, int first, int count) {
    char* sbase = lds + stage * kStage + wave * 8 * 1024;
    const int koff = kt * (BK * 2);
#pragma unroll
    for (int i = first; i < first + count; ++i) {
      if (i < 8)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (lds_void*)(sbase + i * 1024), 16, (int)offA[i], koff, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rB, (lds_void*)(sbase + kOperandStage + (i - 8) * 1024), 16,
                                                 (int)offB[i - 8], koff, 0, 0);
    }
  };

  bf16x8 fa[2][4], fb[2][4];
  auto load_frags = [&](int set, int stage, int kk) {
    const char* s = lds + stage * kStage;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) fa[set][rb] = *(const bf16x8*)(s + aBase + rb * 4096 + roff[kk]);
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) fb[set][cb] = *(const bf16x8*)(s + bBase + cb * 4096 + roff[kk]);
  };
  auto mfmas = [&](int set) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][rb], fb[set][cb], acc[rb][cb], 0, 0, 0);
  };
  const int nk = K / BK;
  issue_range(0, 0, 0, 16);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  block_barrier();
  load_frags(0, 0, 0);
  // loads 0..5 of tile 1 belong to "k-step 3 of the previous tile"; there is none, issue them here
  issue_range(1, min(1, nk - 1), 0, 6);

  for (int kt = 0; kt < nk; ++kt) {
    const int stage = kt & 1;
    const int next_tile = min(kt + 1, nk - 1);   // clamped past the end: refills a stage nobody reads again
    // k-step 0
    __builtin_amdgcn_sched_barrier(0);
    issue_range(stage ^ 1, next_tile, 6, 5);
    load_frags(1, stage, 1);
    mfmas(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i % 2 == 1 || i == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    __builtin_amdgcn_sched_barrier(0);
    // k-step 1
    issue_range(stage ^ 1, next_tile, 11, 5);
    load_frags(0, stage, 2);
    mfmas(1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i % 2 == 1 || i == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    __builtin_amdgcn_sched_barrier(0);
    // k-step 2
    load_frags(1, stage, 3);
    mfmas(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    __builtin_amdgcn_sched_barrier(0);
    // the next tile has landed; every wave is done reading this tile's stage
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    block_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // k-step 3: first fragments of the next tile, first loads of the tile after it
    issue_range(stage, min(kt + 2, nk - 1), 0, 6);
    load_frags(0, stage ^ 1, 0);
    mfmas(1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i % 2 == 1 || i == 0 || i == 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the clamped tail loads before LDS is reused
}

// ---------------------------------------------------------------------------------------
// Probe linear.  Rows = tokens (A = X), columns = out features (B = W).
// Side state first, base GEMM second: the accumulators of a foreground row are
// +0 after the side phase (its side operand rows are zero), i.e. exactly the
// state a plain GEMM starts from, so foreground rows come out bit-identical to
// an all-foreground call.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void k_probe_gemm(ProbeGemmArgs p, int n_tm, int n_tn) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int tm, tn;
  if (!tile_of_block(blockIdx.x, n_tm, n_tn, tm, tn)) return;
  const int tile_m0 = tm * BM, tile_n0 = tn * BN;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, kg = (lane >> 5) * 8;

  f32x16 acc[4][4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;

  if (p.has_side) {
    const int NC = p.RP + p.Rp;
    const int tile_end = min(tile_m0 + BM, p.T);
    int rows[4], cols[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      rows[i] = tile_m0 + wm * 128 + i * 32 + lrow;
      cols[i] = min(tile_n0 + wn * 128 + i * 32 + lrow, p.m - 1);
    }
    // walk the sequences that intersect this row tile
    int s = __builtin_amdgcn_readfirstlane(p.tok_seq[tile_m0]);
    bool any_cand = false;
    while (true) {
      const int seg_lo = max(__builtin_amdgcn_readfirstlane(p.cu[s]), tile_m0);
      const int seq_end = __builtin_amdgcn_readfirstlane(p.cu[s + 1]);
      const int seg_hi = min(seq_end, tile_end);
      const int kind = __builtin_amdgcn_readfirstlane(p.seq_kind[s]);
      if (seg_hi > seg_lo && kind >= kKindCentre) any_cand = true;
      if (seg_hi > seg_lo && kind >= 0) {
        const bf16_t* Ud = p.Uh + (int64_t)kind * p.m * p.RP;
        for (int ks = 0; ks < p.RP; ks += 16) {
          bf16x8 fa[4], fb[4];
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) {
            const bool in = rows[rb] >= seg_lo && rows[rb] < seg_hi;
            fa[rb] = in ? load_frag(p.Aside + (int64_t)rows[rb] * NC + ks + kg) : zero_frag();
          }
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) fb[cb] = load_frag(Ud + (int64_t)cols[cb] * p.RP + ks + kg);
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
              acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[rb], fb[cb], acc[rb][cb], 0, 0, 0);
        }
      }
      if (seq_end >= tile_end || s + 1 >= p.S) break;
      ++s;
    }
    if (any_cand && p.Rp > 0) {
      for (int ks = 0; ks < p.Rp; ks += 16) {
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
          fa[rb] = load_frag(p.Aside + (int64_t)min(rows[rb], p.T - 1) * NC + p.RP + ks + kg);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) fb[cb] = load_frag(p.Ph + (int64_t)cols[cb] * p.Rp + ks + kg);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[rb], fb[cb], acc[rb][cb], 0, 0, 0);
      }
    }
  }

  gemm_mainloop(p.X, p.ldx, p.T, tile_m0, p.W, p.ldw, p.m, tile_n0, p.n, acc, lds);

  // epilogue: D[i][j], i = 8*(v/4) + 4*(lane/32) + v%4, j = lane%32
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    const int col = tile_n0 + wn * 128 + cb * 32 + lrow;
    if (col >= p.m) continue;
    const float bias = p.bias ? p.bias[col] : 0.0f;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = tile_m0 + wm * 128 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row >= p.T) continue;
        float y = acc[rb][cb][v];
        if (p.bias) y += bias;
        if (p.act == 1) y = fmaxf(y, 0.0f);
        if (p.out_bf16) ((bf16_t*)p.Y)[(int64_t)row * p.ldy + col] = f32_to_bf16(y);
        else ((float*)p.Y)[(int64_t)row * p.ldy + col] = y;
      }
    }
  }
}

hipError_t launch_probe_gemm_bf16(const ProbeGemmArgs& a, hipStream_t st) {
  if (a.T == 0 || a.m == 0) return hipSuccess;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)k_probe_gemm, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_tm = (a.T + BM - 1) / BM, n_tn = (a.m + BN - 1) / BN;
  const int total = n_tm * n_tn;
  const int grid = ((total + kXcds - 1) / kXcds) * kXcds;
  hipLaunchKernelGGL(k_probe_gemm, dim3(grid), dim3(256), kGemmLds, st, a, n_tm, n_tn);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Fused LM-head scoring.  Rows = vocabulary (A = W_head), columns = tokens
// (B = H), so that a lane holds 16 logits of ONE token per 32x32 block and the
// log-sum-exp reduction over the vocabulary is mostly in-register.  Each
// workgroup emits, per token of its tile, the maximum logit and
// sum exp(z - max) over its 256 vocabulary rows, and the target logit if the
// target falls in the tile.  Logits are never written.
// ---------------------------------------------------------------------------------------
int head_vocab_tiles_bf16(int vocab) { return (vocab + BM - 1) / BM; }

__global__ __launch_bounds__(256, 1) void k_head_score(HeadScoreArgs p, int n_tm, int n_tn) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int tm, tn;
  if (!tile_of_block(blockIdx.x, n_tm, n_tn, tm, tn)) return;
  const int tile_v0 = tm * BM, tile_t0 = tn * BN;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, lhalf = lane >> 5;

  f32x16 acc[4][4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;

  gemm_mainloop(p.Wh, p.ldw, p.vocab, tile_v0, p.H, p.ldh, p.T, tile_t0, p.d, acc, lds);

  __syncthreads();  // every wave is done reading operand tiles; reuse LDS for the exchange
  float* s_max = (float*)lds;          // [2][256]
  float* s_sum = s_max + 2 * BN;       // [2][256]
  constexpr float kLog2e = 1.4426950408889634f;
  const int vbase = tile_v0 + wm * 128;  // first vocabulary row of this wave

#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    const int tl = wn * 128 + cb * 32 + lrow;   // token within the tile
    const int t = tile_t0 + tl;
    float mx = -INFINITY;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int vr = vbase + rb * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
        if (vr >= p.vocab) acc[rb][cb][v] = -INFINITY;
        mx = fmaxf(mx, acc[rb][cb][v]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mref = (mx == -INFINITY) ? 0.0f : mx;
    float sum = 0.0f;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f((acc[rb][cb][v] - mref) * kLog2e);
    sum += __shfl_xor(sum, 32);
    if (lhalf == 0) { s_max[wm * BN + tl] = mx; s_sum[wm * BN + tl] = sum; }
    // target logit: exactly one lane of the whole grid holds it
    if (t < p.T) {
      const int loc = p.targets[t] - vbase;
      if (loc >= 0 && loc < 128 && ((loc >> 2) & 1) == lhalf) {
        const int sel = (loc >> 5) * 16 + ((loc & 31) >> 3) * 4 + (loc & 3);
        float z = 0.0f;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (sel == rb * 16 + v) z = acc[rb][cb][v];
        p.tgt_logit[t] = z;
      }
    }
  }
  __syncthreads();
  {
    const int t = tile_t0 + tid;
    if (t < p.T) {
      const float m0 = s_max[tid], m1 = s_max[BN + tid];
      const float M = fmaxf(m0, m1);
      const float mref = (M == -INFINITY) ? 0.0f : M;
      const float S = s_sum[tid] * __builtin_amdgcn_exp2f((m0 - mref) * kLog2e) +
                      s_sum[BN + tid] * __builtin_amdgcn_exp2f((m1 - mref) * kLog2e);
      p.part_max[(int64_t)tm * p.T + t] = M;
      p.part_sum[(int64_t)tm * p.T + t] = S;
    }
  }
}

hipError_t launch_head_score_bf16(const HeadScoreArgs& a, hipStream_t st) {
  if (a.T == 0) return hipSuccess;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)k_head_score, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_tm = (a.vocab + BM - 1) / BM, n_tn = (a.T + BN - 1) / BN;
  const int total = n_tm * n_tn;
  const int grid = ((total + kXcds - 1) / kXcds) * kXcds;
  hipLaunchKernelGGL(k_head_score, dim3(grid), dim3(256), kGemmLds, st, a, n_tm, n_tn);
  return hipGetLastError();
}

}  // namespace zo
