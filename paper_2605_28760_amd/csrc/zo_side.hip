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
  // The grid is sized for the worst case (most items, largest k-split); the k-split and the number
  // of items are known on the device.  Block b is (group b / ksplit, split b % ksplit), so the blocks
  // without work are the last ones of the grid and are dispatched after every block that has some.
  const int n_items = a.n_items[0];
  const int ksplit = a.n_items[1];
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

  const bool fg = it.kind == kKindForeground;
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
        if (cb == 0 && !kDir) continue;
        const int col = cb == 0 ? lr : ndir_cols + (cb0 + cb - 1) * 16 + lr;
        const float x = acc[rb][cb][v];
        if (ksplit == 1) {
          float y = x;
          if (cb == 0) y = has_dir ? it.scale * x : 0.0f;
          if (fg) y = 0.0f;
          a.Aside[row * NC + col] = f32_to_bf16(y);
        } else if (!fg) {   // the reduction kernel writes the zeros of foreground rows without reading partials
          a.partial[((int64_t)split * a.T + row) * NC + col] = x;
        }
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
  const int ksplit = a.n_items[1];
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
  f32x4 acc[4][NDB];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int b = 0; b < NDB; ++b) acc[rb][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (has_dir) {
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
      for (int b = 0; b < NDB; ++b) {
        const int col = (cbd0 + b) * 16 + lr;
        if (ksplit == 1) a.Aside[row * NC + col] = f32_to_bf16(has_dir ? it.scale * acc[rb][b][v] : 0.0f);
        else a.partial[((int64_t)split * a.T + row) * NC + col] = acc[rb][b][v];
      }
    }
}

// Fixed-order sum of the k-split partials, scaling and rounding to bf16.  Without a split the
// side-down pass has written Aside itself.
__global__ void k_side_reduce(SideDownArgs a) {
  const int ksplit = a.n_items[1];
  if (ksplit == 1) return;
  const int NC = a.RP + a.Rp;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)a.T * NC) return;
  const int row = (int)(idx / NC), col = (int)(idx % NC);
  const int s = a.tok_seq[row];
  const int kind = a.seq_kind[s];
  float y = 0.0f;
  const bool live = (col < a.RP) ? (kind >= 0) : (kind >= kKindCentre);
  if (live) {
    for (int sp = 0; sp < ksplit; ++sp) y += a.partial[((int64_t)sp * a.T + row) * NC + col];
    if (col < a.RP) y *= a.seq_scale[s];
  }
  a.Aside[idx] = f32_to_bf16(y);
}

template <int NBB, bool kDir>
static void launch_pass(const SideDownArgs& a, int cb0, hipStream_t st) {
  dim3 grid(a.ks_cap * ((a.max_items + 3) / 4));
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
    dim3 grid(a.ks_cap * ((a.max_items + 3) / 4));
    const int left = a.RP / 16 - cbd;
    if (left >= 8) { hipLaunchKernelGGL(k_side_down_dirblocks<8>, grid, dim3(256), 0, st, a, cbd); cbd += 8; }
    else if (left >= 4) { hipLaunchKernelGGL(k_side_down_dirblocks<4>, grid, dim3(256), 0, st, a, cbd); cbd += 4; }
    else if (left >= 2) { hipLaunchKernelGGL(k_side_down_dirblocks<2>, grid, dim3(256), 0, st, a, cbd); cbd += 2; }
    else { hipLaunchKernelGGL(k_side_down_dirblocks<1>, grid, dim3(256), 0, st, a, cbd); cbd += 1; }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.ks_cap > 1) {
    const int64_t total = (int64_t)a.T * (a.RP + a.Rp);
    hipLaunchKernelGGL(k_side_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace zo
