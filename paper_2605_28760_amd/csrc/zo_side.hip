// Side-down projection: the "A = V^T" half of the LoRA-style side state of
// Sec. 3.2.  For every candidate row t it forms
//     [ X[t,:] V_{k_t}  |  X[t,:] Vb ]
// as fp32 partial sums over a few K ranges; a finishing kernel sums the ranges,
// scales the direction part by s_t eps, rounds to bf16 and lays the rows out as
// the token-side operand of the probe GEMM's side K tiles, which multiply them
// by [U_{k_t} | P]^T.  The pass streams X once and is bound by HBM bandwidth;
// the skinny contraction runs on v_mfma_f32_16x16x32_bf16 so that the
// arithmetic (about 2 (r + R) flop per byte of X) stays out of the way.
//
// Work items are chunks of at most 64 (or 48, 32 or 16: the host picks the size
// that fills the chip in the fewest rounds of workgroups) rows of one candidate
// sequence, so all rows of an item share one direction; foreground sequences
// have no items.  One wave per (item, K range); the seven or eight waves of a
// workgroup walk the same K range in steps of 64 columns, so the bank operand
// Vb is staged once per workgroup in LDS.  A wave's rows of X land in
// its own two-stage ring in LDS (direct-to-LDS loads of whole 128-byte lines,
// no registers tied up by bytes in flight): while a wave multiplies step s, the
// lines of steps s+1 and s+2 are on their way.
#include <type_traits>

#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

typedef __attribute__((address_space(3))) void lds_void;
constexpr int kNonTemporal = 2;   // cache-policy operand of a buffer load: the nt bit

// 16x16x32 bf16 MFMA: A fragment = 16 rows x 32 k (lane l: row l%16, k = 8*(l/16)..+7),
// B fragment = 32 k x 16 cols (lane l: col l%16, same k), D: lane l holds rows 4*(l/16)+v, col l%16.
// Here the columns of V take the A side and the rows of X the B side: D[column of V][row of X].
//
// NBB = number of 16-column bank blocks this pass accumulates (cb0 = the first of them); kDir = whether
// the pass also carries the first 16-column direction block; RB = 16-row blocks of an item.
//
// LDS: [wave][2 stages][RB*16 rows][128 B] rings of X, then [2 stages][NBB blocks][2 halves][1 KiB] of Vb,
// then [wave][2 KiB] for each wave's direction block of V (one stage).
// A row of a ring stage holds its eight 16-byte chunks XOR-swizzled by (row >> 1) & 7, which makes the
// fragment reads (16 rows x 4 chunks per instruction) conflict-free.
//
// One step of a wave: wait for the step's lines (leaving the next step's in flight), barrier (the
// step's Vb stage is complete, and every wave is done with the other stage), request the next step's
// Vb stage, read the step's X and V fragments into registers, then multiply, with the requests for the
// next step's V block and for the lines of the step after next (into the ring stage just read) spread
// through the products.
template <int NBB, bool kDir, int RB, int W>
__global__ __launch_bounds__(W * 64, 1) void k_side_down(SideDownArgs a, int cb0) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr int kRing = RB * 2048;                   // one ring stage: RB*16 rows x 128 B
  constexpr int kVbStage = (NBB > 0 ? NBB : 1) * 2048;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  char* ring = lds + wave * 2 * kRing;
  char* s_vb = lds + W * 2 * kRing;
  char* s_vd = s_vb + 2 * kVbStage + wave * 2048;   // this wave's direction block of V: one stage
  // The grid is sized for the largest possible number of items; their number is known on the device.
  // Block b is (group b / ksplit, split b % ksplit), so the blocks without work are the last ones of the
  // grid and are dispatched after every block that has some.
  const int n_items = a.n_items[0];
  const int ksplit = a.ksplit;
  const int group = blockIdx.x / ksplit, split = blockIdx.x - group * ksplit;
  if (group * W >= n_items) return;
  const int item_raw = group * W + wave;
  const bool live = item_raw < n_items;
  // waves without an item still take part in the workgroup's Vb loads and barriers
  SideItem it = a.items[live ? item_raw : n_items - 1];
  it.row0 = __builtin_amdgcn_readfirstlane(it.row0);
  it.nrows = __builtin_amdgcn_readfirstlane(it.nrows);
  it.kind = __builtin_amdgcn_readfirstlane(it.kind);
  const int NC = a.RP + a.Rp;
  const int lr = lane & 15, lg = lane >> 4;
  // each split walks its own contiguous K range in steps of 64; the first (steps mod k-split) splits
  // take one step more
  constexpr int kstride = 64;
  const int steps_total = a.n / kstride;
  const int q = steps_total / ksplit, rem = steps_total - q * ksplit;
  const int k_begin = (split * q + min(split, rem)) * kstride;
  const int nsteps_all = q + (split < rem ? 1 : 0);
  const bool has_dir = kDir && it.kind >= 0;
  // wave-uniform.  (The item list holds no foreground sequences: their rows have no side term and are not
  // read at all; the finishing kernel writes their zeros.)
  const bool work = live;
  const int nsteps = nsteps_all;

  // X -> ring: load j (0 .. 2*RB-1) covers rows 8j .. 8j+7; lane i lands at byte 16*i of its 1 KiB block:
  // row 8j + i/8, physical chunk i%8 = logical chunk ^ ((row >> 1) & 7).  Rows past the item's end repeat
  // its last row (their results are never stored).
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.X + (int64_t)it.row0 * a.ldx), 0,
      (int)min(((int64_t)(it.nrows - 1) * a.ldx + a.n) * 2, (int64_t)0x7FFFFFFF), 0x00020000);
  uint32_t x_off[2 * RB];
#pragma unroll
  for (int j = 0; j < 2 * RB; ++j) {
    const int row = 8 * j + (lane >> 3);
    const int lch = (lane & 7) ^ ((row >> 1) & 7);
    x_off[j] = (uint32_t)min(row, it.nrows - 1) * (uint32_t)(a.ldx * 2) + (uint32_t)(k_begin * 2 + lch * 16);
  }
  // load j of the step's rows of X (non-temporal: a line of X is used once, and should not push V and Vb
  // out of the L2)
  auto issue_x1 = [&](int step, int j) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (lds_void*)(ring + (step & 1) * kRing + j * 1024), 16, (int)x_off[j],
                                             step * kstride * 2, 0, kNonTemporal);
  };
  auto issue_x = [&](int step) {
    if (!work) return;
#pragma unroll
    for (int j = 0; j < 2 * RB; ++j) issue_x1(step, j);
  };
  // fragment (rb, h) of a ring stage: row rb*16 + lr, logical chunk h*4 + lg
  uint32_t a_off[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) a_off[h] = lr * 128 + (((h * 4 + lg) ^ ((lr >> 1) & 7)) << 4);

  // Vb -> LDS: load j (0 .. 2*NBB-1) = (half h = j & 1, block b = j >> 1); lane i fills byte 16*i of
  // the 1 KiB block: col i/4, physical chunk i%4 = logical chunk ^ ((col>>2)&3)
  const int vcol = lane >> 2;
  const int vchunk = (lane & 3) ^ ((vcol >> 2) & 3);
  const uint32_t vb_off = (uint32_t)((int64_t)vcol * a.n + k_begin + vchunk * 8) * 2u;
  const __amdgpu_buffer_rsrc_t vb_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.Vbt + (int64_t)cb0 * 16 * a.n), 0, (int)((int64_t)(NBB > 0 ? NBB : 1) * 16 * a.n * 2), 0x00020000);
  const uint32_t rd_off = lr * 64 + ((lg ^ ((lr >> 2) & 3)) << 4);
  constexpr int kVbMine = (2 * NBB + W - 1) / W;   // Vb loads of one wave per step (at most)
  auto issue_vb = [&](int step) {
    char* dst = s_vb + (step & 1) * kVbStage;
#pragma unroll
    for (int i = 0; i < kVbMine; ++i) {
      const int j = wave + i * W;
      if (j < 2 * NBB) {
        const int h = j & 1, b = j >> 1;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(vb_rsrc, (lds_void*)(dst + (h * NBB + b) * 1024), 16, (int)vb_off,
                                                 (b * 16 * a.n + step * kstride + h * 32) * 2, 0, 0);
      }
    }
  };
  // The item's own direction block of V^T goes through LDS as well, in the layout of a Vb block.  (No load of
  // the loop returns into registers: for those the compiler places its own waits, and it counts the
  // direct-to-LDS loads in flight as done, so such a wait would drain the whole prefetch.)  A centre item
  // has no direction: it reads direction 0's block and discards the result.
  const __amdgpu_buffer_rsrc_t vd_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.Vt + (int64_t)(has_dir ? it.kind : 0) * a.RP * a.n), 0, (int)((int64_t)16 * a.n * 2), 0x00020000);
  auto issue_v1 = [&](int step, int h) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(vd_rsrc, (lds_void*)(s_vd + h * 1024), 16, (int)vb_off,
                                             (step * kstride + h * 32) * 2, 0, 0);
  };
  auto issue_v = [&](int step) {
    if (!kDir || !work) return;
#pragma unroll
    for (int h = 0; h < 2; ++h) issue_v1(step, h);
  };

  f32x4 acc[RB][NBB + 1];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < NBB + 1; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // In program order a wave requests: X(0) Vb(0) V(0) X(1), then per step s: Vb(s+1) V(s+1) X(s+2).
  // Memory returns in order, so "at most the 2*RB loads of X(s+1) outstanding" means step s has landed.
  if (nsteps > 0) {
    issue_x(0);
    if (NBB > 0) issue_vb(0);
    issue_v(0);
    if (nsteps > 1) issue_x(1);
  }
  for (int step = 0; step < nsteps; ++step) {
    if (step + 1 < nsteps && work) {
      if constexpr (RB == 4) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if constexpr (RB == 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
      else if constexpr (RB == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    // (a bare barrier: __syncthreads() would also wait for every load in flight, the next step's included)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (step + 1 < nsteps && NBB > 0) issue_vb(step + 1);
    bf16x8 fa[2][RB], fv[2];
    if (work) {
      const char* st = ring + (step & 1) * kRing;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) fa[h][rb] = *(const bf16x8*)(st + rb * 2048 + a_off[h]);
        if (kDir) fv[h] = *(const bf16x8*)(s_vd + h * 1024 + rd_off);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // both have been read: they can take what comes next
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) fa[h][rb] = zero_frag();
        fv[h] = zero_frag();
      }
    }
    // The requests for V(s+1) and X(s+2) are spread through the products, one after each group of them:
    // a wave that issued them in one burst would stand at the memory pipeline's queue while its matrix
    // instructions wait behind them in program order.  (Their order, V before X, is what the count of the
    // wait above relies on.)
    const bool more_v = kDir && work && step + 1 < nsteps, more_x = work && step + 2 < nsteps;
    constexpr int kSlots = 2 * (NBB + (kDir ? 1 : 0));      // groups of products in a step
    constexpr int kLoads = (kDir ? 2 : 0) + 2 * RB;          // requests of a step: V halves, then X row blocks
    auto issue_slot = [&](int slot) {
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        if (i * kSlots / kLoads != slot) continue;
        if (kDir && i < 2) {
          if (more_v) issue_v1(step + 1, i);
        } else {
          if (more_x) issue_x1(step + 2, i - (kDir ? 2 : 0));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    // The Vb fragments of the first half are all read before the first product; a fragment of the second
    // half is read as soon as its slot's first-half fragment has been handed to the matrix core, so the
    // latency of an LDS read is paid once per step, not once per fragment.
    const char* stage = s_vb + (step & 1) * kVbStage;
    bf16x8 cur[NBB > 0 ? NBB : 1];
#pragma unroll
    for (int b = 0; b < NBB; ++b) cur[b] = *(const bf16x8*)(stage + b * 1024 + rd_off);
    __builtin_amdgcn_sched_barrier(0);
    int slot = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int b = 0; b < NBB; ++b) {
        const bf16x8 fb = cur[b];
        if (h == 0) cur[b] = *(const bf16x8*)(stage + (NBB + b) * 1024 + rd_off);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc[rb][b + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb, fa[h][rb], acc[rb][b + 1], 0, 0, 0);
        issue_slot(slot++);
      }
      if (kDir) {
        if (work) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fv[h], fa[h][rb], acc[rb][0], 0, 0, 0);
        }
        issue_slot(slot++);
      }
    }
  }
  if (!live) return;

  // (the direction columns of a centre item get no partial sums: the finishing kernel does not read them)
  // The products are formed with the columns of V as the matrix instruction's rows and the rows of X as its
  // columns, so a lane holds four neighbouring columns of one row: one 16-byte store each.
  const int ndir_cols = a.RP;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int lrow = rb * 16 + lr;
    if (lrow >= it.nrows) continue;
    float* dst = a.partial + ((int64_t)split * a.T + it.row0 + lrow) * NC + lg * 4;
#pragma unroll
    for (int cb = 0; cb < NBB + 1; ++cb) {
      if (cb == 0 && (!kDir || !has_dir)) continue;
      const int col = cb == 0 ? 0 : ndir_cols + (cb0 + cb - 1) * 16;
      *reinterpret_cast<f32x4*>(dst + col) = acc[rb][cb];
    }
  }
  // direction columns 16 .. RP-1 exist only for ranks above 16 and are handled by extra passes below
}

// Direction blocks beyond the first (ranks above 16): the same walk over X with no bank blocks, NDB
// 16-column blocks of the item's own V per pass (blocks cbd0 .. cbd0 + NDB - 1).
template <int NDB>
__global__ __launch_bounds__(256) void k_side_down_dirblocks(SideDownArgs a, int cbd0) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ksplit = a.ksplit;
  const int group = blockIdx.x / ksplit, split = blockIdx.x - group * ksplit;
  const int item = group * 4 + wave;
  if (item >= a.n_items[0]) return;
  const SideItem it = a.items[item];
  const int NC = a.RP + a.Rp;
  const int lr = lane & 15, lg = lane >> 4;
  const int steps_total = a.n / 64;
  const int q = steps_total / ksplit, rem = steps_total - q * ksplit;
  const int k_begin = (split * q + min(split, rem)) * 64, kchunk = (q + (split < rem ? 1 : 0)) * 64;
  const bool has_dir = it.kind >= 0;
  if (!has_dir) return;   // centre and foreground rows have no direction columns
  f32x4 acc[4][NDB];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int b = 0; b < NDB; ++b) acc[rb][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  {
    const bf16_t* pv = a.Vt + ((int64_t)it.kind * a.RP + cbd0 * 16 + lr) * a.n + k_begin + lg * 8;
    const bf16_t* pa[4];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
      pa[rb] = a.X + (int64_t)(it.row0 + min(rb * 16 + lr, it.nrows - 1)) * a.ldx + k_begin + lg * 8;
    for (int k = 0; k < kchunk; k += 32) {
      bf16x8 fa[4], fb[NDB];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) fa[rb] = load_frag(pa[rb] + k);
#pragma unroll
      for (int b = 0; b < NDB; ++b) fb[b] = load_frag(pv + (int64_t)b * 16 * a.n + k);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int b = 0; b < NDB; ++b)
          acc[rb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[rb], fb[b], acc[rb][b], 0, 0, 0);
    }
  }
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int lrow = rb * 16 + lg * 4 + v;
      if (lrow >= it.nrows) continue;
      const int64_t row = it.row0 + lrow;
#pragma unroll
      for (int b = 0; b < NDB; ++b)
        a.partial[((int64_t)split * a.T + row) * NC + (cbd0 + b) * 16 + lr] = acc[rb][b][v];
    }
}

// Finishes the side-down pass: sums the K-range partials of every candidate row in range order, scales the
// direction columns by sign * eps, rounds to bf16 and writes the token-side images of the GEMM's side K
// tiles: pool K tile p = [256 rows of its token tile][64 columns].  Direction K tile j of a tile holds the
// slots 2j and 2j+1 (32 columns each): a row has its own direction's block there and zeros in every other
// slot; the bank K tiles follow.  Rows of foreground sequences, rows past the end of the batch and unused
// columns are zero.  One workgroup per (pool K tile, 32 rows); a thread writes 8 columns (16 bytes).
__global__ __launch_bounds__(256) void k_side_finish(SideDownArgs a) {
  const int p = blockIdx.x >> 3;
  if (p >= a.n_items[1]) return;
  const int tn = a.kt_tile[p];
  const TileHdr h = a.tile_hdr[tn];
  const int j = p - h.kt0;
  const int rr = (blockIdx.x & 7) * 32 + (threadIdx.x >> 3), c = threadIdx.x & 7;
  const int row = tn * kTileN + rr;
  const int NC = a.RP + a.Rp;
  const int n_dir_kt = (h.n_slots + 1) >> 1;
  float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (row < a.T) {
    const int s = a.tok_seq[row];
    const int kind = a.seq_kind[s];
    int col = -1, ncol = 0;   // first partial column behind this thread's 8 values, how many of them exist
    float scale = 1.0f;
    if (j < n_dir_kt) {
      const int slot = 2 * j + (c >> 2);
      if (kind >= 0 && slot < h.n_slots) {
        const int e = a.tile_slots[h.slot0 + slot];
        if (e / a.SPD == kind) {
          col = (e % a.SPD) * 32 + (c & 3) * 8;
          ncol = min(8, a.RP - col);
          scale = a.seq_scale[s];
        }
      }
    } else if (kind >= kKindCentre) {
      const int bcol = (j - n_dir_kt) * 64 + c * 8;
      col = a.RP + bcol;
      ncol = min(8, a.Rp - bcol);
    }
    if (ncol > 0) {
      for (int sp = 0; sp < a.ksplit; ++sp) {
        const float4* src = reinterpret_cast<const float4*>(a.partial + ((int64_t)sp * a.T + row) * NC + col);
        const float4 u = src[0], w = src[1];   // RP and Rp are multiples of 16: all 8 exist
        y[0] += u.x; y[1] += u.y; y[2] += u.z; y[3] += u.w;
        y[4] += w.x; y[5] += w.y; y[6] += w.z; y[7] += w.w;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] *= scale;
    }
  }
  u32x4 out = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])};
  *reinterpret_cast<u32x4*>(a.Xs + ((int64_t)p * kTileN + rr) * kTileK + c * 8) = out;
}

template <int NBB, bool kDir, int RB>
static hipError_t launch_pass_rb(const SideDownArgs& a, int cb0, hipStream_t st) {
  constexpr int W = side_waves_of(NBB, RB);
  constexpr int lds_bytes = side_lds_bytes(NBB, RB, W);
  static_assert(lds_bytes <= 160 * 1024, "side-down LDS layout exceeds a compute unit's LDS");
  static std::atomic<bool> configured[kMaxDevices];
  const hipError_t ec = once_per_device(configured, [] {
    return hipFuncSetAttribute((const void*)k_side_down<NBB, kDir, RB, W>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  });
  if (ec != hipSuccess) return ec;
  dim3 grid(a.ksplit * ((a.max_items + W - 1) / W));
  hipLaunchKernelGGL((k_side_down<NBB, kDir, RB, W>), grid, dim3(W * 64), lds_bytes, st, a, cb0);
  return hipGetLastError();
}

template <int NBB, bool kDir>
static hipError_t launch_pass(const SideDownArgs& a, int cb0, hipStream_t st) {
  if (a.item_rows > 48) return launch_pass_rb<NBB, kDir, 4>(a, cb0, st);
  if (a.item_rows > 32) return launch_pass_rb<NBB, kDir, 3>(a, cb0, st);
  if (a.item_rows > 16) return launch_pass_rb<NBB, kDir, 2>(a, cb0, st);
  return launch_pass_rb<NBB, kDir, 1>(a, cb0, st);
}

template <bool kDir>
static hipError_t launch_pass_n(int nbb, const SideDownArgs& a, int cb0, hipStream_t st) {
  switch (nbb) {
    case 0: return launch_pass<0, kDir>(a, cb0, st);
    case 1: return launch_pass<1, kDir>(a, cb0, st);
    case 2: return launch_pass<2, kDir>(a, cb0, st);
    case 3: return launch_pass<3, kDir>(a, cb0, st);
    case 4: return launch_pass<4, kDir>(a, cb0, st);
    case 5: return launch_pass<5, kDir>(a, cb0, st);
    case 6: return launch_pass<6, kDir>(a, cb0, st);
    case 7: return launch_pass<7, kDir>(a, cb0, st);
    default: return launch_pass<8, kDir>(a, cb0, st);
  }
}

hipError_t launch_side_down_bf16(const SideDownArgs& a, hipStream_t st) {
  if (a.T == 0 || a.max_items == 0) return hipSuccess;
  const int bank_blocks = a.Rp / 16;
  // first pass: direction block 0 together with up to 8 bank blocks
  int done = bank_blocks < kSideMaxBlocks - 1 ? bank_blocks : kSideMaxBlocks - 1;
  hipError_t e0 = launch_pass_n<true>(done, a, 0, st);
  if (e0 != hipSuccess) return e0;
  while (done < bank_blocks) {   // bank ranks above 128: further passes over X
    const int nb = bank_blocks - done < kSideMaxBlocks - 1 ? bank_blocks - done : kSideMaxBlocks - 1;
    e0 = launch_pass_n<false>(nb, a, done, st);
    if (e0 != hipSuccess) return e0;
    done += nb;
  }
  for (int cbd = 1; cbd < a.RP / 16;) {   // ranks above 16: up to 8 further direction blocks per pass over X
    dim3 grid(a.ksplit * ((a.max_items + 3) / 4));
    const int left = a.RP / 16 - cbd;
    if (left >= 8) { hipLaunchKernelGGL(k_side_down_dirblocks<8>, grid, dim3(256), 0, st, a, cbd); cbd += 8; }
    else if (left >= 4) { hipLaunchKernelGGL(k_side_down_dirblocks<4>, grid, dim3(256), 0, st, a, cbd); cbd += 4; }
    else if (left >= 2) { hipLaunchKernelGGL(k_side_down_dirblocks<2>, grid, dim3(256), 0, st, a, cbd); cbd += 2; }
    else { hipLaunchKernelGGL(k_side_down_dirblocks<1>, grid, dim3(256), 0, st, a, cbd); cbd += 1; }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_side_finish, dim3((unsigned)a.kt_cap * 8u), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace zo
