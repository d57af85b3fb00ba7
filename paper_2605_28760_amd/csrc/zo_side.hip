// Side-down projection: the "A = V^T" half of the LoRA-style side state of
// Sec. 3.2.  For every candidate row t it forms
//     Aside[t, :] = [ s_t eps (X[t,:] V_{k_t})  |  X[t,:] Vb ]        (bf16)
// which the probe GEMM then multiplies by [U_{k_t} | P]^T.  The kernel streams
// X once and is bound by HBM bandwidth; the skinny contraction runs on
// v_mfma_f32_16x16x32_bf16 so that the arithmetic (about 2 (r + R) flop per
// byte of X) stays out of the way.
//
// Work items are chunks of at most 64 rows of one sequence, so all rows of an
// item share one direction.  One wave per (item, k-split); the four waves of a
// workgroup walk the same K range, so the bank operand Vb is staged once per
// workgroup in LDS (direct-to-LDS loads, double buffered) while each wave keeps
// its own rows of X and its own direction's V in registers.
#include <type_traits>

#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

typedef __attribute__((address_space(3))) void lds_void;

// 16x16x32 bf16 MFMA: A fragment = 16 rows x 32 k (lane l: row l%16, k = 8*(l/16)..+7),
// B fragment = 32 k x 16 cols (lane l: col l%16, same k), D: lane l holds rows 4*(l/16)+v, col l%16.
//
// NBB = number of 16-column bank blocks this pass accumulates; kDir = whether the pass
// also carries the (single) 16-column direction block.  cb0 = first bank block of the pass.
//
// One K step of 64: a wave issues the loads of its 64 rows (8 KiB) and of its direction's V, the
// workgroup's Vb slice goes to one of two alternating LDS stages, everybody waits, one barrier,
// multiply.  Measured alternatives on this part: keeping a second step of X in flight in registers
// is slower (3.0 against 4.3 TB/s: the loads of a step already fill the memory pipeline), as are
// steps of 32 or 128, items of 16 or 32 rows, and a third workgroup per CU (register spills).
template <int NBB, bool kDir>
__global__ __launch_bounds__(256, 2) void k_side_down(SideDownArgs a, int cb0) {
  // Vb stage: [half h of the K step][16-col block][col][4 chunks of 16 B], chunk index XOR (col>>2)&3
  __shared__ __attribute__((aligned(1024))) char s_vb[2][NBB > 0 ? NBB * 2048 : 16];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  // The grid is sized for the largest possible number of items; their number is known on the device.
  // Block b is (group b / ksplit, split b % ksplit), so the blocks without work are the last ones of the
  // grid and are dispatched after every block that has some.
  const int n_items = a.n_items[0];
  const int ksplit = a.ksplit;
  const int group = blockIdx.x / ksplit, split = blockIdx.x - group * ksplit;
  if (group * 4 >= n_items) return;
  const int item_raw = group * 4 + wave;
  const bool live = item_raw < n_items;
  // waves without an item still take part in the workgroup's Vb loads and barriers
  const SideItem it = a.items[live ? item_raw : n_items - 1];
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
  const bool work = live && it.kind != kKindForeground;   // wave-uniform; foreground rows are not read at all
  // a workgroup whose four items are all foreground (or absent) has nothing to multiply: it skips the
  // K loop and only writes its zeros
  const bool wg_work = __syncthreads_or(work) != 0;

  // per-lane addresses: 16 B at (row, k + h*32 + lg*8)
  const bf16_t* pa[4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const int row = it.row0 + min(rb * 16 + lr, it.nrows - 1);
    pa[rb] = a.X + (int64_t)row * a.ldx + k_begin + lg * 8;
  }
  // a centre item has no direction: read a valid address (its own X rows), discard the result
  const bf16_t* pv = has_dir ? a.Vt + ((int64_t)it.kind * a.RP + lr) * a.n + k_begin + lg * 8 : pa[0];
  // Vb -> LDS: load j (0 .. 2*NBB-1) = (half h = j & 1, block b = j >> 1); lane i fills byte 16*i of
  // the 1 KiB block: col i/4, physical chunk i%4 = logical chunk ^ ((col>>2)&3)
  const int vcol = lane >> 2;
  const int vchunk = (lane & 3) ^ ((vcol >> 2) & 3);
  // (buffer loads: rows of Vbt from bank column cb0*16 on; the byte offset of this lane's first piece)
  const uint32_t vb_off = (uint32_t)((int64_t)vcol * a.n + k_begin + vchunk * 8) * 2u;
  const __amdgpu_buffer_rsrc_t vb_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.Vbt + (int64_t)cb0 * 16 * a.n), 0, (int)((int64_t)(NBB > 0 ? NBB : 1) * 16 * a.n * 2), 0x00020000);
  const uint32_t rd_off = lr * 64 + ((lg ^ ((lr >> 2) & 3)) << 4);

  auto issue_vb = [&](int stage, int step) {
#pragma unroll
    for (int j = 0; j < 2 * NBB; ++j) {
      if ((j & 3) != wave) continue;
      const int h = j & 1, b = j >> 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vb_rsrc, (lds_void*)(&s_vb[stage][0] + (h * NBB + b) * 1024), 16,
                                               (int)vb_off, (b * 16 * a.n + step * kstride + h * 32) * 2, 0, 0);
    }
  };

  f32x4 acc[4][NBB + 1];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int cb = 0; cb < NBB + 1; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Refilling stage (step+1)&1 is safe once a wave is past barrier `step`: every wave has then
  // finished the MFMAs of step-1, the last reader of that stage.
  const int nsteps = wg_work ? nsteps_all : 0;
  for (int step = 0; step < nsteps; ++step) {
    bf16x8 fa[2][4], fv[2];   // [half][row block], [half]
    if (work) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) fa[h][rb] = load_frag(pa[rb] + step * kstride + h * 32);
        if (kDir) fv[h] = load_frag(pv + step * kstride + h * 32);
      }
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) fa[h][rb] = zero_frag();
        fv[h] = zero_frag();
      }
    }
    if (NBB > 0) issue_vb(step & 1, step);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const char* stage = &s_vb[step & 1][0];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      bf16x8 fb[NBB > 0 ? NBB : 1];
#pragma unroll
      for (int b = 0; b < NBB; ++b) fb[b] = *(const bf16x8*)(stage + (h * NBB + b) * 1024 + rd_off);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        if (kDir) acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[h][rb], fv[h], acc[rb][0], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < NBB; ++b)
          acc[rb][b + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[h][rb], fb[b], acc[rb][b + 1], 0, 0, 0);
      }
    }
  }
  if (!live) return;

  // Rows of foreground sequences get no partial sums: the finishing kernel writes their zeros without
  // reading any.  Neither do the direction columns of a centre item.
  if (it.kind == kKindForeground) return;
  const int ndir_cols = a.RP;
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int lrow = rb * 16 + lg * 4 + v;
      if (lrow >= it.nrows) continue;
      const int64_t row = it.row0 + lrow;
#pragma unroll
      for (int cb = 0; cb < NBB + 1; ++cb) {
        if (cb == 0 && (!kDir || !has_dir)) continue;
        const int col = cb == 0 ? lr : ndir_cols + (cb0 + cb - 1) * 16 + lr;
        a.partial[((int64_t)split * a.T + row) * NC + col] = acc[rb][cb][v];
      }
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

template <int NBB, bool kDir>
static void launch_pass(const SideDownArgs& a, int cb0, hipStream_t st) {
  dim3 grid(a.ksplit * ((a.max_items + 3) / 4));
  hipLaunchKernelGGL((k_side_down<NBB, kDir>), grid, dim3(256), 0, st, a, cb0);
}

template <bool kDir>
static void launch_pass_n(int nbb, const SideDownArgs& a, int cb0, hipStream_t st) {
  switch (nbb) {
    case 0: launch_pass<0, kDir>(a, cb0, st); break;
    case 1: launch_pass<1, kDir>(a, cb0, st); break;
    case 2: launch_pass<2, kDir>(a, cb0, st); break;
    case 3: launch_pass<3, kDir>(a, cb0, st); break;
    case 4: launch_pass<4, kDir>(a, cb0, st); break;
    case 5: launch_pass<5, kDir>(a, cb0, st); break;
    case 6: launch_pass<6, kDir>(a, cb0, st); break;
    case 7: launch_pass<7, kDir>(a, cb0, st); break;
    default: launch_pass<8, kDir>(a, cb0, st); break;
  }
}

hipError_t launch_side_down_bf16(const SideDownArgs& a, hipStream_t st) {
  if (a.T == 0 || a.max_items == 0) return hipSuccess;
  const int bank_blocks = a.Rp / 16;
  // first pass: direction block 0 together with up to 8 bank blocks
  int done = bank_blocks < kSideMaxBlocks - 1 ? bank_blocks : kSideMaxBlocks - 1;
  launch_pass_n<true>(done, a, 0, st);
  while (done < bank_blocks) {   // bank ranks above 128: further passes over X
    const int nb = bank_blocks - done < kSideMaxBlocks - 1 ? bank_blocks - done : kSideMaxBlocks - 1;
    launch_pass_n<false>(nb, a, done, st);
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

// K ranges per row: ranges of about 2560 columns for wide inputs, four ranges up to 8192 columns, never
// narrower than 512 columns, whole 64-column steps.
int side_ksplit(int n) {
  int s = n <= 8192 ? 4 : (n + 1280) / 2560;
  if (s > 8) s = 8;
  while (s > 1 && n / s < 512) --s;
  return s < 1 ? 1 : s;
}

}  // namespace zo
