// Matrix-core kernels for gfx950: the probe linear (Sec. 3.2: every candidate
// row sees W_0 + s eps U V^T + P Vb^T, applied as factors) and the fused
// LM-head scoring (Sec. 3.3: per-request NLL without materialising logits).
//
// Both are one persistent 256x256x64-tiled bf16 GEMM with fp32 accumulation on
// v_mfma_f32_32x32x16_bf16.  One workgroup per CU; four waves in a 2x2 grid own
// 128x128 each.  MFMA rows are the rows of the weight matrix (out features /
// vocabulary), MFMA columns are tokens: a lane then holds 16 weight-row values
// of ONE token per 32x32 block, which keeps the vocabulary reduction of the
// head in registers and packs probe outputs into contiguous bf16.
//
// Operand tiles stream global -> LDS with direct-to-LDS buffer loads into a
// double-buffered, XOR-swizzled layout.  The stream of K tiles does not stop at
// the end of an output tile: while a tile's epilogue runs, the first K tiles of
// the workgroup's next output tile are already landing.  Workgroups walk a
// grouped raster so that the 32 workgroups resident on one XCD share an 8x4
// block of output tiles in that XCD's L2.
//
// Determinism / batch invariance: the tile shape and the K order never depend
// on the batch, there is no split-K and no atomic, so a token's result depends
// only on that token's operands.
#include <type_traits>

#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {

constexpr int BM = kTileM, BN = kTileN, BK = kTileK;
constexpr int kOperandStage = BM * BK * 2;        // 32 KiB: one operand tile (256 rows x 128 B)
constexpr int kStage = 2 * kOperandStage;         // A tile then B tile
constexpr int kStagesLds = 2 * kStage;            // double buffered operand stages: 128 KiB
constexpr int kEpiLds = 32 * 1024;                // epilogue scratch, disjoint from the stages
constexpr int kGemmLds = kStagesLds + kEpiLds;    // 160 KiB: the whole LDS of a CU
constexpr int kGroupM = 8;                        // raster: weight-row tiles per group
constexpr int kXcds = 8;
#ifndef ZO_HEAD_WAVES
#define ZO_HEAD_WAVES 4
#endif

typedef __attribute__((address_space(3))) void lds_void;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 __attribute__((may_alias)) u32x2_alias;   // LDS staging is written and read back with different widths
typedef u32x4 __attribute__((may_alias)) u32x4_alias;

// Position L of the grouped raster -> output tile (tm = weight-row tile, tn = token tile).
__device__ __forceinline__ void tile_at(int L, int n_tm, int n_tn, int& tm, int& tn) {
  const int per_group = kGroupM * n_tn;
  const int g = L / per_group, in_g = L - g * per_group;
  const int first_m = g * kGroupM;
  const int gsize = min(n_tm - first_m, kGroupM);
  tm = first_m + in_g % gsize;
  tn = in_g / gsize;
}

__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Per-lane addressing of one output tile's operand stream.  Load j (0..7) of a wave
// fills the 1 KiB block (wave*8 + j) of an operand tile: 8 rows x 128 B.  Lane i lands at
// byte 16*i of the block, i.e. row i/8, physical chunk i%8, which holds logical chunk
// (i%8) ^ ((row>>1)&7).  Rows past the end of a matrix are clamped to its last row (their
// results are never stored); the buffer resources bound every access to the matrix anyway.
template <int LPW>   // loads per wave per operand tile (8 with four waves, 4 with eight)
struct OperandStream {
  __amdgpu_buffer_rsrc_t rA, rB;
  uint32_t offA[LPW], offB[LPW];
};

template <int LPW>
__device__ __forceinline__ void setup_stream(OperandStream<LPW>& o, const bf16_t* A, int64_t lda, int M, int tile_m0,
                                             const bf16_t* B, int64_t ldb, int N, int tile_n0, int K, int wave,
                                             int lane) {
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int row = (wave * LPW + j) * 8 + (lane >> 3);
    const int lch = (lane & 7) ^ ((row >> 1) & 7);
    const int ra = min(tile_m0 + row, M - 1) - tile_m0;
    const int rbn = min(tile_n0 + row, N - 1) - tile_n0;
    o.offA[j] = (uint32_t)((int64_t)ra * lda * 2 + lch * 16);
    o.offB[j] = (uint32_t)((int64_t)rbn * ldb * 2 + lch * 16);
  }
  const int64_t bytesA = ((int64_t)(M - tile_m0 - 1) * lda + K) * 2;
  const int64_t bytesB = ((int64_t)(N - tile_n0 - 1) * ldb + K) * 2;
  o.rA = __builtin_amdgcn_make_buffer_rsrc((void*)(A + (int64_t)tile_m0 * lda), 0,
                                           (int)min(bytesA, (int64_t)0x7FFFFFFF), 0x00020000);
  o.rB = __builtin_amdgcn_make_buffer_rsrc((void*)(B + (int64_t)tile_n0 * ldb), 0,
                                           (int)min(bytesB, (int64_t)0x7FFFFFFF), 0x00020000);
}

// Persistent GEMM driver.  For every output tile of this workgroup:
//   pre(tm, tn, acc)   may add side terms into the zeroed accumulators,
//   acc[rb][cb] += A[tile rows] * B[tile rows]^T over K (multiple of 64),
//   post(tm, tn, acc)  consumes the accumulators (it may use lds + kStagesLds .. +kEpiLds
//                      and workgroup barriers; it must not touch the operand stages).
//
// Pipeline of the K loop.  K tiles of 64 (128-byte row segments, so every L2 request is a
// full line) alternate between two LDS stages.  A K tile is four k-steps of 16; MFMA
// fragments are double buffered in registers and the LDS reads of the next k-step run
// under the 16 MFMAs of the current one.  The 16 direct-to-LDS loads a wave issues per
// K tile are spread thinly (one per ~3 MFMAs) over k-step 3 of the previous K tile and
// k-steps 0..1 of the current one: a burst would fill the memory pipeline's queues and
// stall the wave, and with it the MFMA stream.  The single barrier of a K tile sits before
// k-step 3: by then every wave has read its last fragments of this K tile's stage (so the
// stage can be refilled) and the next K tile has landed (so its first fragments can be
// fetched under k-step 3).  The load cursor runs ahead of the compute cursor across
// output-tile boundaries; past the workgroup's last tile it stays on the final K tile
// (those loads refill stages nobody reads again).
// Wave layouts.  WAVES = 4: 2x2 waves of 128x128 (one wave per SIMD, all 256 accumulators of a
// lane in use).  WAVES = 8: 2x4 waves of 128 weight rows x 64 tokens (two waves per SIMD: while
// one wave is held up issuing a memory instruction the other keeps the matrix core fed, at the
// price of 1.5x the LDS fragment reads).
template <int WAVES>
struct WaveShape {
  static constexpr int kWN = WAVES / 2;            // waves along tokens
  static constexpr int kRB = 4;                    // 32-row blocks per wave (128 weight rows)
  static constexpr int kCB = (BN / kWN) / 32;      // 32-token blocks per wave (4 or 2)
  static constexpr int kLPW = 32 / WAVES;          // loads per wave per operand tile
};

template <int WAVES, class Pre, class Post>
__device__ __forceinline__ void persistent_gemm(const bf16_t* __restrict__ A, int64_t lda, int M,
                                                const bf16_t* __restrict__ B, int64_t ldb, int N, int K,
                                                int n_tm, int n_tn, char* lds, Pre pre, Post post) {
  using WS = WaveShape<WAVES>;
  constexpr int RB = WS::kRB, CB = WS::kCB, LPW = WS::kLPW;
  constexpr int NL = 2 * LPW;                      // loads per wave per K tile
  constexpr int L3 = (NL * 3 + 7) / 8, L0 = (NL - L3 + 1) / 2, L1 = NL - L3 - L0;   // 16 -> 6,5,5;  8 -> 3,3,2
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave / WS::kWN, wn = wave % WS::kWN;

  // this workgroup's tiles: positions first, first + stride, ... of its XCD's share of the raster
  const int total = n_tm * n_tn;
  const int per_xcd = (total + kXcds - 1) / kXcds;
  const int xcd = blockIdx.x % kXcds;
  const int stride = gridDim.x / kXcds;
  const int L_end = min((xcd + 1) * per_xcd, total);
  int L = xcd * per_xcd + blockIdx.x / kXcds;
  if (L >= L_end) return;
  const int nk = K / BK;

  // LDS -> register mapping (32x32x16 fragments: lane l holds row l%32, k-group l/32)
  const int lrow = lane & 31;
  const int swz = (lrow >> 1) & 7;
  uint32_t roff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) roff[kk] = lrow * 128 + (((kk * 2 + (lane >> 5)) ^ swz) << 4);
  const uint32_t aBase = wm * 128 * 128, bBase = kOperandStage + wn * (CB * 32) * 128;

  // load cursor
  OperandStream<LPW> ld;
  int ld_L = L, ld_kt = 0;
  {
    int tm, tn;
    tile_at(ld_L, n_tm, n_tn, tm, tn);
    setup_stream(ld, A, lda, M, tm * BM, B, ldb, N, tn * BN, K, wave, lane);
  }
  // load i (0..NL-1) of the cursor's K tile: i < LPW -> A chunk i, else B chunk i - LPW
  auto issue_range = [&](int stage, int first, int count) {
    char* sbase = lds + stage * kStage + wave * LPW * 1024;
    const int koff = ld_kt * (BK * 2);
#pragma unroll
    for (int i = first; i < first + count; ++i) {
      if (i < LPW)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rA, (lds_void*)(sbase + i * 1024), 16, (int)ld.offA[i], koff, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rB, (lds_void*)(sbase + kOperandStage + (i - LPW) * 1024), 16,
                                                 (int)ld.offB[i - LPW], koff, 0, 0);
    }
  };
  auto advance_cursor = [&]() {
    if (ld_kt + 1 < nk) { ++ld_kt; return; }
    if (ld_L + stride < L_end) {
      ld_L += stride;
      ld_kt = 0;
      int tm, tn;
      tile_at(ld_L, n_tm, n_tn, tm, tn);
      setup_stream(ld, A, lda, M, tm * BM, B, ldb, N, tn * BN, K, wave, lane);
    }
  };

  bf16x8 fa[2][RB], fb[2][CB];
  auto load_frags = [&](int set, int stage, int kk) {
    const char* s = lds + stage * kStage;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) fa[set][rb] = *(const bf16x8*)(s + aBase + rb * 4096 + roff[kk]);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) fb[set][cb] = *(const bf16x8*)(s + bBase + cb * 4096 + roff[kk]);
  };
  // scheduling of one k-step: the RB+CB LDS reads and `loads` direct-to-LDS loads go under the
  // first MFMAs (one read per MFMA, a load after every other one), the rest of the MFMAs follow
  auto pattern = [&](auto loads_tag) {
    constexpr int loads = decltype(loads_tag)::value;
#pragma unroll
    for (int i = 0; i < RB + CB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
      if (i < loads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // direct-to-LDS load
    }
    __builtin_amdgcn_sched_group_barrier(0x008, RB * CB - (RB + CB), 0);
  };

  // prologue: first K tile of the first output tile, and the head of the second K tile
  issue_range(0, 0, NL);
  advance_cursor();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  block_barrier();
  load_frags(0, 0, 0);
  issue_range(1, 0, L3);

  int stage = 0;
  for (; L < L_end; L += stride) {
    int tm, tn;
    tile_at(L, n_tm, n_tn, tm, tn);
    f32x16 acc[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;
    pre(tm, tn, acc);

    auto mfmas = [&](int set) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][rb], fb[set][cb], acc[rb][cb], 0, 0, 0);
    };

    for (int kt = 0; kt < nk; ++kt) {
      // k-step 0
      __builtin_amdgcn_sched_barrier(0);
      issue_range(stage ^ 1, L3, L0);
      load_frags(1, stage, 1);
      mfmas(0);
      pattern(std::integral_constant<int, L0>{});
      __builtin_amdgcn_sched_barrier(0);
      // k-step 1
      issue_range(stage ^ 1, L3 + L0, L1);
      load_frags(0, stage, 2);
      mfmas(1);
      pattern(std::integral_constant<int, L1>{});
      __builtin_amdgcn_sched_barrier(0);
      // k-step 2
      load_frags(1, stage, 3);
      mfmas(0);
      pattern(std::integral_constant<int, 0>{});
      __builtin_amdgcn_sched_barrier(0);
      // the next K tile has landed; every wave is done reading this K tile's stage
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      block_barrier();
      advance_cursor();
      __builtin_amdgcn_sched_barrier(0);
      // k-step 3: first fragments of the next K tile, first loads of the one after it
      issue_range(stage, 0, L3);
      load_frags(0, stage ^ 1, 0);
      mfmas(1);
      pattern(std::integral_constant<int, L3>{});
      __builtin_amdgcn_sched_barrier(0);
      stage ^= 1;
    }
    post(tm, tn, acc);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the trailing loads before the workgroup ends
}

static int gemm_grid(int total_tiles) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < kXcds)
      n = 256;
    cus = n;
  }
  const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
  const int slots = per_xcd < cus / kXcds ? per_xcd : cus / kXcds;
  return slots * kXcds;
}

// ---------------------------------------------------------------------------------------
// Probe linear.  Side state first, base GEMM second: the accumulators of a foreground
// token are +0 after the side phase (its side operand rows are zero), i.e. exactly the
// state a plain GEMM starts from, so foreground rows come out bit-identical to an
// all-foreground call.
// ---------------------------------------------------------------------------------------
template <bool kSide, bool kOutBf16, bool kBias>
__global__ __launch_bounds__(256, 1) void k_probe_gemm(ProbeGemmArgs p, int n_tm, int n_tn) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = lane & 31, lhalf = lane >> 5, kg = lhalf * 8;

  auto side_phase = [&](int tm, int tn, f32x16 (&acc)[4][4]) {
    if constexpr (!kSide) return;
    const int tile_o0 = tm * BM, tile_t0 = tn * BN;
    const int NC = p.RP + p.Rp;
    const int tile_end = min(tile_t0 + BN, p.T);
    int feat[4], tok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      feat[i] = min(tile_o0 + wm * 128 + i * 32 + lrow, p.m - 1);
      tok[i] = tile_t0 + wn * 128 + i * 32 + lrow;
    }
    // walk the sequences that intersect this token tile
    int s = __builtin_amdgcn_readfirstlane(p.tok_seq[tile_t0]);
    bool any_cand = false;
    while (true) {
      const int seg_lo = max(__builtin_amdgcn_readfirstlane(p.cu[s]), tile_t0);
      const int seq_end = __builtin_amdgcn_readfirstlane(p.cu[s + 1]);
      const int seg_hi = min(seq_end, tile_end);
      const int kind = __builtin_amdgcn_readfirstlane(p.seq_kind[s]);
      if (seg_hi > seg_lo && kind >= kKindCentre) any_cand = true;
      if (seg_hi > seg_lo && kind >= 0) {
        const bf16_t* Ud = p.Uh + (int64_t)kind * p.m * p.RP;
        for (int ks = 0; ks < p.RP; ks += 16) {
          bf16x8 fa[4], fb[4];
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) fa[rb] = load_frag(Ud + (int64_t)feat[rb] * p.RP + ks + kg);
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) {
            const bool in = tok[cb] >= seg_lo && tok[cb] < seg_hi;
            fb[cb] = in ? load_frag(p.Aside + (int64_t)tok[cb] * NC + ks + kg) : zero_frag();
          }
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
        for (int rb = 0; rb < 4; ++rb) fa[rb] = load_frag(p.Ph + (int64_t)feat[rb] * p.Rp + ks + kg);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
          fb[cb] = load_frag(p.Aside + (int64_t)min(tok[cb], p.T - 1) * NC + p.RP + ks + kg);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[rb], fb[cb], acc[rb][cb], 0, 0, 0);
      }
    }
  };

  // D[i][j]: i = 8*(v/4) + 4*(lane/32) + v%4 (out feature), j = lane%32 (token).
  auto epilogue = [&](int tm, int tn, f32x16 (&acc)[4][4]) {
    const int obase = tm * BM + wm * 128;   // first out feature of this wave
    const int tbase = tn * BN + wn * 128;   // first token of this wave
    if constexpr (!kOutBf16) {
      float* Y = (float*)p.Y;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int t = tbase + cb * 32 + lrow;
        if (t >= p.T) continue;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int o = obase + rb * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
            if (o >= p.m) continue;
            float y = acc[rb][cb][v];
            if constexpr (kBias) y += p.bias[o];
            if (p.act == 1) y = fmaxf(y, 0.0f);
            Y[(int64_t)t * p.ldy + o] = y;
          }
      }
      return;
    }
    // bf16: bias / activation / rounding in registers, then 32 tokens x 128 features at a
    // time through this wave's own 8 KiB of LDS (XOR-swizzled 16-byte slots) so that the
    // global stores are 16 bytes per lane and cover 256 contiguous bytes per token row.
    char* region = lds + kStagesLds + wave * 8192;
    bf16_t* Y = (bf16_t*)p.Y;
    const int chunk = lane & 15;              // 8 out features (16 bytes) of a token row
    const int o = obase + chunk * 8;
    const float floor_val = p.act == 1 ? 0.0f : -INFINITY;   // ReLU as a clamp: no branch in the tile epilogue
    const uint32_t wr_base = lrow * 256 + lhalf * 8;
    const uint32_t wr_swz = (lrow & 15) * 16;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = acc[rb][cb][g * 4 + e];
          if constexpr (kBias) {
            const int ob = obase + rb * 32 + 8 * g + 4 * lhalf;   // this lane's 4 consecutive out features
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] += p.bias[min(ob + e, p.m - 1)];
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = fmaxf(y[e], floor_val);
          *(u32x2_alias*)(region + wr_base + (((rb * 4 + g) * 16) ^ wr_swz)) =
              u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
        }
      }
      // the wave reads back what it wrote itself: LDS operations of one wave complete in order
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int tl = it * 4 + (lane >> 4);
        const int t = tbase + cb * 32 + tl;
        const u32x4 val = *(const u32x4_alias*)(region + tl * 256 + ((chunk ^ (tl & 15)) * 16));
        if (t < p.T && o < p.m) *(u32x4_alias*)(Y + (int64_t)t * p.ldy + o) = val;   // m % 8 == 0
      }
    }
  };

  persistent_gemm<4>(p.W, p.ldw, p.m, p.X, p.ldx, p.T, p.n, n_tm, n_tn, lds, side_phase, epilogue);
}

template <bool kSide, bool kOutBf16, bool kBias>
static hipError_t launch_probe_variant(const ProbeGemmArgs& a, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)k_probe_gemm<kSide, kOutBf16, kBias>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_tm = (a.m + BM - 1) / BM, n_tn = (a.T + BN - 1) / BN;
  hipLaunchKernelGGL((k_probe_gemm<kSide, kOutBf16, kBias>), dim3(gemm_grid(n_tm * n_tn)), dim3(256), kGemmLds, st,
                     a, n_tm, n_tn);
  return hipGetLastError();
}

template <bool kSide, bool kOutBf16>
static hipError_t launch_probe_bias(const ProbeGemmArgs& a, hipStream_t st) {
  return a.bias ? launch_probe_variant<kSide, kOutBf16, true>(a, st) : launch_probe_variant<kSide, kOutBf16, false>(a, st);
}

hipError_t launch_probe_gemm_bf16(const ProbeGemmArgs& a, hipStream_t st) {
  if (a.T == 0 || a.m == 0) return hipSuccess;
  if (a.has_side) return a.out_bf16 ? launch_probe_bias<true, true>(a, st) : launch_probe_bias<true, false>(a, st);
  return a.out_bf16 ? launch_probe_bias<false, true>(a, st) : launch_probe_bias<false, false>(a, st);
}

// ---------------------------------------------------------------------------------------
// Fused LM-head scoring.  Each output tile emits, per token, the maximum logit and
// sum exp(z - max) over its 256 vocabulary rows, and the target logit if the target
// falls in the tile.  Logits are never written.
// ---------------------------------------------------------------------------------------
int head_vocab_tiles_bf16(int vocab) { return (vocab + BM - 1) / BM; }

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, 1) void k_head_score(HeadScoreArgs p, int n_tm, int n_tn) {
  using WS = WaveShape<WAVES>;
  constexpr int CB = WS::kCB;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave / WS::kWN, wn = wave % WS::kWN;
  const int lrow = lane & 31, lhalf = lane >> 5;
  float* s_max = (float*)(lds + kStagesLds);   // [2][256]
  float* s_sum = s_max + 2 * BN;                // [2][256]
  constexpr float kLog2e = 1.4426950408889634f;

  auto no_side = [](int, int, f32x16 (&)[4][CB]) {};
  auto epilogue = [&](int tm, int tn, f32x16 (&acc)[4][CB]) {
    const int tile_v0 = tm * BM, tile_t0 = tn * BN;
    const int vbase = tile_v0 + wm * 128;  // first vocabulary row of this wave
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const int tl = wn * (CB * 32) + cb * 32 + lrow;   // token within the tile
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
      if (tid < BN && t < p.T) {
        const float m0 = s_max[tid], m1 = s_max[BN + tid];
        const float Mx = fmaxf(m0, m1);
        const float mref = (Mx == -INFINITY) ? 0.0f : Mx;
        const float S = s_sum[tid] * __builtin_amdgcn_exp2f((m0 - mref) * kLog2e) +
                        s_sum[BN + tid] * __builtin_amdgcn_exp2f((m1 - mref) * kLog2e);
        p.part_max[(int64_t)tm * p.T + t] = Mx;
        p.part_sum[(int64_t)tm * p.T + t] = S;
      }
    }
    __syncthreads();   // the exchange buffers are free again for the next tile
  };

  persistent_gemm<WAVES>(p.Wh, p.ldw, p.vocab, p.H, p.ldh, p.T, p.d, n_tm, n_tn, lds, no_side, epilogue);
}

constexpr int kHeadWaves = ZO_HEAD_WAVES;

hipError_t launch_head_score_bf16(const HeadScoreArgs& a, hipStream_t st) {
  if (a.T == 0) return hipSuccess;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)k_head_score<kHeadWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_tm = (a.vocab + BM - 1) / BM, n_tn = (a.T + BN - 1) / BN;
  hipLaunchKernelGGL((k_head_score<kHeadWaves>), dim3(gemm_grid(n_tm * n_tn)), dim3(kHeadWaves * 64), kGemmLds, st, a, n_tm, n_tn);
  return hipGetLastError();
}

}  // namespace zo
