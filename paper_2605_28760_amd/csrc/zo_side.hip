// Side-down projection: the "A = V^T" half of the LoRA-style side state of
// Sec. 3.2.  For every candidate row t it forms
//     Aside[t, :] = [ s_t eps (X[t,:] V_{k_t})  |  X[t,:] Vb ]        (bf16)
// which the probe GEMM then multiplies by [U_{k_t} | P]^T.  The kernel streams
// X once (it is bound by HBM bandwidth); work items are chunks of one
// sequence, so all rows of an item share one direction.
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

// One wave per (item, k-split).  16x16x32 bf16 MFMA: A fragment = 16 rows x 32 k
// (lane l: row l%16, k = 8*(l/16)..+7), B fragment = 32 k x 16 cols (lane l: col
// l%16, same k), D: lane l holds rows 4*(l/16)+v, col l%16.
template <int NB>
__global__ __launch_bounds__(256) void k_side_down(SideDownArgs a, int cb0) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + wave;
  const int n_items = *a.n_items;
  if (item >= n_items) return;
  const SideItem it = a.items[item];
  const int split = blockIdx.y;
  const int NC = a.RP + a.Rp;
  const int lr = lane & 15, lg = lane >> 4;
  const int ndir_blocks = a.RP >> 4;

  if (it.kind == kKindForeground) {
    if (a.ksplit == 1) {
      for (int idx = lane; idx < it.nrows * NB * 16; idx += 64) {
        const int row = idx / (NB * 16), c = idx % (NB * 16);
        a.Aside[(int64_t)(it.row0 + row) * NC + cb0 * 16 + c] = 0;
      }
    }
    return;
  }

  const int kchunk = a.n / a.ksplit;
  const int k_begin = split * kchunk;

  const bf16_t* pa[4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const int row = it.row0 + min(rb * 16 + lr, it.nrows - 1);
    pa[rb] = a.X + (int64_t)row * a.ldx + k_begin + lg * 8;
  }
  const bf16_t* pb[NB];
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) {
    const int gcb = cb0 + cb;
    if (gcb < ndir_blocks) {
      // a centre item has no direction: read a valid address (its own X rows) and discard the result
      pb[cb] = it.kind >= 0 ? a.Vt + ((int64_t)it.kind * a.RP + gcb * 16 + lr) * a.n + k_begin + lg * 8 : pa[0];
    } else {
      pb[cb] = a.Vbt + ((int64_t)(gcb - ndir_blocks) * 16 + lr) * a.n + k_begin + lg * 8;
    }
  }

  f32x4 acc[4][NB];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};


  for (int k = 0; k < kchunk; k += 32) {
    bf16x8 fa[4], fb[NB];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) fa[rb] = load_frag(pa[rb] + k);
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) fb[cb] = load_frag(pb[cb] + k);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int cb = 0; cb < NB; ++cb)
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[rb], fb[cb], acc[rb][cb], 0, 0, 0);
  }

#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int lrow = rb * 16 + lg * 4 + v;
      if (lrow >= it.nrows) continue;
      const int64_t row = it.row0 + lrow;
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
        const int gcb = cb0 + cb;
        const int col = gcb * 16 + lr;
        const float x = acc[rb][cb][v];
        if (a.ksplit == 1) {
          float y = x;
          if (gcb < ndir_blocks) y = (it.kind >= 0) ? it.scale * x : 0.0f;
          a.Aside[row * NC + col] = f32_to_bf16(y);
        } else {
          a.partial[((int64_t)split * a.T + row) * NC + col] = x;
        }
      }
    }
  }
}

// Fixed-order sum of the k-split partials, scaling and rounding to bf16.
__global__ void k_side_reduce(SideDownArgs a) {
  const int NC = a.RP + a.Rp;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)a.T * NC) return;
  const int row = (int)(idx / NC), col = (int)(idx % NC);
  const int s = a.tok_seq[row];
  const int kind = a.seq_kind[s];
  float y = 0.0f;
  const bool live = (col < a.RP) ? (kind >= 0) : (kind >= kKindCentre);
  if (live) {
    for (int sp = 0; sp < a.ksplit; ++sp) y += a.partial[((int64_t)sp * a.T + row) * NC + col];
    if (col < a.RP) y *= a.seq_scale[s];
  }
  a.Aside[idx] = f32_to_bf16(y);
}

template <int NB>
static void launch_pass(const SideDownArgs& a, int cb0, hipStream_t st) {
  dim3 grid((a.max_items + 3) / 4, a.ksplit);
  hipLaunchKernelGGL(k_side_down<NB>, grid, dim3(256), 0, st, a, cb0);
}

hipError_t launch_side_down_bf16(const SideDownArgs& a, hipStream_t st) {
  if (a.T == 0 || a.max_items == 0) return hipSuccess;
  const int nblocks = (a.RP + a.Rp) / 16;
  for (int cb0 = 0; cb0 < nblocks; cb0 += kSideMaxBlocks) {
    const int nb = nblocks - cb0 < kSideMaxBlocks ? nblocks - cb0 : kSideMaxBlocks;
    switch (nb) {
      case 1: launch_pass<1>(a, cb0, st); break;
      case 2: launch_pass<2>(a, cb0, st); break;
      case 3: launch_pass<3>(a, cb0, st); break;
      case 4: launch_pass<4>(a, cb0, st); break;
      case 5: launch_pass<5>(a, cb0, st); break;
      case 6: launch_pass<6>(a, cb0, st); break;
      case 7: launch_pass<7>(a, cb0, st); break;
      case 8: launch_pass<8>(a, cb0, st); break;
      default: launch_pass<9>(a, cb0, st); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (a.ksplit > 1) {
    const int64_t total = (int64_t)a.T * (a.RP + a.Rp);
    hipLaunchKernelGGL(k_side_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace zo
