// Folding the bank into the base (Sec. 3.2: standalone runs may fold the external state;
// Eq. "bank" read right to left):  W[i][j] += sum_k P[i][k] Vb[j][k] over the R columns in
// use, then those columns are cleared.  The bank is fp32 and the only rounding that may
// matter is the one into W's storage type, so the product runs on the fp32 matrix
// instruction (v_mfma_f32_32x32x2_f32: exact fp32 products, fp32 accumulation).  The pass
// reads and writes W once; at the paper's ranks (64..512) it is bound by HBM up to rank
// 64 and by the fp32 matrix rate above.
#include <type_traits>

#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {
namespace {

typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int kFoldRows = 32;     // rows of W per wave (one MFMA tile high)
constexpr int kFoldCols = 128;    // columns of W per wave (four MFMA tiles wide)
constexpr int kFoldWaves = 4;     // a workgroup covers 128 x 128
constexpr int kFoldTile = kFoldWaves * kFoldRows;
constexpr int kFoldK = 32;        // bank columns staged per step
constexpr int kFoldKPitch = kFoldK + 4;     // floats per staged operand row: 16-byte reads of 32 rows hit every bank equally
constexpr int kFoldStage = 64;    // columns of W staged through LDS at a time in the epilogue
constexpr int kFoldPitch = kFoldStage + 4;  // floats per staged output row
constexpr int kFoldOperandFloats = 2 * kFoldTile * kFoldKPitch;            // P panel + Vb panel
constexpr int kFoldEpilogueFloats = kFoldWaves * kFoldRows * kFoldPitch;   // one region per wave
constexpr int kFoldLdsFloats = kFoldOperandFloats > kFoldEpilogueFloats ? kFoldOperandFloats : kFoldEpilogueFloats;

// One row segment of 4 bank columns [k, k+4) of row `row` of a [rows x R_cap] matrix, zero outside the
// matrix or past the R columns in use.
__device__ __forceinline__ float4 fold_operand(const float* A, int rows, int R_cap, int R, int row, int k, int vec_ok) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (row >= rows || k >= R) return v;
  const float* p = A + (int64_t)row * R_cap + k;
  if (vec_ok && k + 4 <= R) return *reinterpret_cast<const float4*>(p);
  v.x = p[0];
  if (k + 1 < R) v.y = p[1];
  if (k + 2 < R) v.z = p[2];
  if (k + 3 < R) v.w = p[3];
  return v;
}

// The four waves of a workgroup share a 128-column panel of Vb and each own 32 rows of P; both
// panels go global -> LDS in row-contiguous 16-byte pieces, 32 bank columns per step.
// Lane l supplies A[row l%32][k-slot l/32] and B[k-slot l/32][column l%32] of a 32x32x2 step and
// receives D[8*(v/4) + 4*(l/32) + v%4][l%32], v = 0..15.  Which bank column sits in which k-slot
// is free as long as A and B agree: of every 8 columns the lower half-wave takes the first 4 and
// the upper the last 4, so a lane fetches its four values with one 16-byte LDS read.  The
// accumulators hold a W tile column-wise per lane; they are staged through a per-wave LDS
// region so that W itself is read and written in 16-byte (bf16) / 32-byte (fp32) row segments.
template <bool kBf16>
__global__ __launch_bounds__(kFoldWaves* kWave, 2) void k_fold_bank(FoldArgs p, int vec_w, int vec_bank) {
  __shared__ __attribute__((aligned(16))) float s_mem[kFoldLdsFloats];   // 36 KiB
  float* s_p = s_mem;
  float* s_v = s_mem + kFoldTile * kFoldKPitch;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jl = lane & 31, h = lane >> 5;
  const int M0 = blockIdx.y * kFoldTile, n0 = blockIdx.x * kFoldCols;
  const int m0 = M0 + wave * kFoldRows;
  f32x16 acc[4];
#pragma unroll
  for (int jt = 0; jt < 4; ++jt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[jt][v] = 0.f;
  // The old values of W are requested first so that they arrive under the product.  Pass (half, it) of
  // the epilogue handles row it*8 + lane/8 and the 8 columns half*64 + (lane%8)*8 of the wave's tile.
  typedef typename std::conditional<kBf16, u32x4, f32x8>::type old_t;
  old_t w_old[kFoldCols / kFoldStage][kFoldRows / 8];
  if (vec_w && m0 < p.m) {
#pragma unroll
    for (int half = 0; half < kFoldCols / kFoldStage; ++half)
#pragma unroll
      for (int it = 0; it < kFoldRows / 8; ++it) {
        const int grow = m0 + it * 8 + (lane >> 3), gcol = n0 + half * kFoldStage + (lane & 7) * 8;
        if (grow < p.m && gcol + 8 <= p.n) {
          const int64_t at = (int64_t)grow * p.ldw + gcol;
          if constexpr (kBf16) w_old[half][it] = *reinterpret_cast<const old_t*>((const bf16_t*)p.W + at);
          else w_old[half][it] = *reinterpret_cast<const old_t*>((const float*)p.W + at);
        }
      }
  }
  // A thread moves 4 + 4 row segments per step; the next step's segments are requested before the
  // product of the current step, so they travel under it.
  constexpr int kSegs = kFoldTile * (kFoldK / 4) / (kFoldWaves * kWave);
  float4 seg_p[kSegs], seg_v[kSegs];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < kSegs; ++i) {
      const int idx = threadIdx.x + i * kFoldWaves * kWave;
      const int row = idx >> 3, seg = idx & 7;
      seg_p[i] = fold_operand(p.P, p.m, p.R_cap, p.R, M0 + row, k0 + seg * 4, vec_bank);
      seg_v[i] = fold_operand(p.Vb, p.n, p.R_cap, p.R, n0 + row, k0 + seg * 4, vec_bank);
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < p.R; k0 += kFoldK) {
#pragma unroll
    for (int i = 0; i < kSegs; ++i) {
      const int idx = threadIdx.x + i * kFoldWaves * kWave;
      const int row = idx >> 3, seg = idx & 7;
      *reinterpret_cast<float4*>(s_p + row * kFoldKPitch + seg * 4) = seg_p[i];
      *reinterpret_cast<float4*>(s_v + row * kFoldKPitch + seg * 4) = seg_v[i];
    }
    __syncthreads();
    if (k0 + kFoldK < p.R) fetch(k0 + kFoldK);
#pragma unroll
    for (int sub = 0; sub < kFoldK / 8; ++sub) {
      const int kk = sub * 8 + 4 * h;
      const float4 a = *reinterpret_cast<const float4*>(s_p + (wave * kFoldRows + jl) * kFoldKPitch + kk);
      float4 b[4];
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) b[jt] = *reinterpret_cast<const float4*>(s_v + (jt * 32 + jl) * kFoldKPitch + kk);
      // the four accumulators take turns, so that consecutive matrix instructions are independent
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b[jt].x, acc[jt], 0, 0, 0);
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b[jt].y, acc[jt], 0, 0, 0);
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b[jt].z, acc[jt], 0, 0, 0);
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b[jt].w, acc[jt], 0, 0, 0);
    }
    __syncthreads();   // the panels are overwritten by the next step (and by the epilogue staging)
  }
  if (m0 >= p.m) return;   // past the last barrier
  const int vec_ok = vec_w;
  float* sd = s_mem + wave * kFoldRows * kFoldPitch;
#pragma unroll
  for (int half = 0; half < kFoldCols / kFoldStage; ++half) {
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        sd[(8 * (v >> 2) + 4 * h + (v & 3)) * kFoldPitch + jt * 32 + jl] = acc[2 * half + jt][v];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    // 8 rows per pass, 8 lanes per row, 8 consecutive columns per lane
#pragma unroll
    for (int it = 0; it < kFoldRows / 8; ++it) {
      const int row = it * 8 + (lane >> 3), col = (lane & 7) * 8;
      const int grow = m0 + row, gcol = n0 + half * kFoldStage + col;
      if (grow >= p.m || gcol >= p.n) continue;
      const float4 d0 = *reinterpret_cast<const float4*>(sd + row * kFoldPitch + col);
      const float4 d1 = *reinterpret_cast<const float4*>(sd + row * kFoldPitch + col + 4);
      const float d[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
      const int64_t at = (int64_t)grow * p.ldw + gcol;
      if constexpr (kBf16) {
        bf16_t* W = (bf16_t*)p.W + at;
        if (vec_ok && gcol + 8 <= p.n) {
          const u32x4 old = w_old[half][it];
          u32x4 out;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            out[i] = pack_bf16x2(__uint_as_float(old[i] << 16) + d[2 * i], __uint_as_float(old[i] & 0xFFFF0000u) + d[2 * i + 1]);
          *reinterpret_cast<u32x4*>(W) = out;
        } else {
          for (int i = 0; i < 8 && gcol + i < p.n; ++i) W[i] = f32_to_bf16(bf16_to_f32(W[i]) + d[i]);
        }
      } else {
        float* W = (float*)p.W + at;
        if (vec_ok && gcol + 8 <= p.n) {
          f32x8 w = w_old[half][it];
#pragma unroll
          for (int i = 0; i < 8; ++i) w[i] += d[i];
          *reinterpret_cast<f32x8*>(W) = w;
        } else {
          for (int i = 0; i < 8 && gcol + i < p.n; ++i) W[i] += d[i];
        }
      }
    }
  }
}

// zeroes columns [0, R) of a [rows x R_cap] fp32 matrix (a fill kernel, so that the call can be captured)
__global__ void k_zero_columns(float* A, int rows, int R_cap, int R) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * R) return;
  A[(idx / R) * R_cap + idx % R] = 0.0f;
}

}  // namespace

hipError_t launch_fold_bank(const FoldArgs& a, hipStream_t st) {
  if (a.m == 0 || a.n == 0 || a.R == 0) return hipSuccess;
  const dim3 grid((a.n + kFoldCols - 1) / kFoldCols, (a.m + kFoldTile - 1) / kFoldTile);
  // whole row segments may be moved as 16-byte vectors when every row starts 16-byte aligned
  const int vec_w = ((uintptr_t)a.W & 15u) == 0 && a.ldw % (a.bf16 ? 8 : 4) == 0;
  const int vec_bank = (((uintptr_t)a.P | (uintptr_t)a.Vb) & 15u) == 0 && a.R_cap % 4 == 0;
  if (a.bf16) k_fold_bank<true><<<grid, kFoldWaves * kWave, 0, st>>>(a, vec_w, vec_bank);
  else k_fold_bank<false><<<grid, kFoldWaves * kWave, 0, st>>>(a, vec_w, vec_bank);
  const int64_t np_ = (int64_t)a.m * a.R, nv = (int64_t)a.n * a.R;
  hipLaunchKernelGGL(k_zero_columns, dim3((unsigned)((np_ + 255) / 256)), dim3(256), 0, st, a.P, a.m, a.R_cap, a.R);
  hipLaunchKernelGGL(k_zero_columns, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, st, a.Vb, a.n, a.R_cap, a.R);
  return hipGetLastError();
}

}  // namespace zo
