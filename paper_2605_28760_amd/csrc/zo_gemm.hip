// Matrix-core kernels for gfx950: the probe linear (Sec. 3.2: every candidate
// row sees W_0 + s eps U V^T + P Vb^T, applied as factors) and the fused
// LM-head scoring (Sec. 3.3: per-request NLL without materialising logits).
//
// Both are one persistent 256x256x64-tiled bf16 GEMM with fp32 accumulation on
// v_mfma_f32_16x16x32_bf16.  One workgroup of eight waves per CU (two per
// SIMD); the waves form a 2x4 grid, each owning 128 weight rows x 64 tokens
// (8x4 blocks of 16x16, 128 accumulator registers per lane).  With two waves
// per SIMD the matrix core stays fed while the other wave is held up issuing
// memory instructions, and on this power-limited part the K=32 instruction
// sustains the highest MFMA rate.  MFMA rows are the rows of the weight matrix
// (out features / vocabulary), MFMA columns are tokens: a lane holds 4
// consecutive weight-row values of ONE token per block, which keeps the
// vocabulary reduction of the head in registers and packs probe outputs into
// contiguous bf16.
//
// Operand tiles stream global -> LDS with direct-to-LDS buffer loads into a
// double-buffered, XOR-swizzled layout.  The stream of K tiles does not stop at
// the end of an output tile: while a tile's epilogue runs, the first K tiles of
// the workgroup's next output tile are already landing.  Workgroups walk a
// grouped raster so that the 32 workgroups resident on one XCD share an 8x4
// block of output tiles in that XCD's L2, and the eight XCDs work on
// neighbouring blocks that share their weight rows.
//
// Determinism / batch invariance: the K order of an output element never
// depends on the batch (a tile may be computed whole or as two halves of 128
// weight rows, which changes which wave holds an element, not its arithmetic),
// there is no split-K and no atomic, so a token's result depends only on that
// token's operands.
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
// A half tile (128 A rows) needs 16 + 32 KiB per stage, so three stages fit next to 16 KiB of epilogue scratch
constexpr int kHalfA = (BM / 2) * BK * 2;         // 16 KiB: 128 rows x 128 B
constexpr int kHalfStage = kHalfA + kOperandStage;
constexpr int kHalfStagesLds = 3 * kHalfStage;    // 144 KiB
constexpr int kGroupM = 8;                        // raster: weight-row tiles per group
constexpr int kXcds = 8;
constexpr int kWaves = 8;                         // 2 (weight rows) x 4 (tokens)
constexpr int kThreads = kWaves * 64;
constexpr int RB = 8;                             // 16-row blocks per wave: 128 weight rows
constexpr int CB = 4;                             // 16-token blocks per wave: 64 tokens
constexpr int kLPW = 32 / kWaves;                 // direct-to-LDS loads per wave per operand tile
// All 8 loads of a K tile are issued in the k-step right after the barrier, which gives them a whole
// K-tile period to land (issuing half of them half a period later measured 3-9 % slower).
constexpr int kLoadsLate = 2 * kLPW;                 // loads of a K tile issued in the k-step after the barrier
constexpr int kLoadsEarly = 2 * kLPW - kLoadsLate;   // ... and in the k-step before the next barrier

typedef __attribute__((address_space(3))) void lds_void;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 __attribute__((may_alias)) u32x2_alias;   // LDS staging is written and read back with different widths
typedef u32x4 __attribute__((may_alias)) u32x4_alias;
typedef f32x4 Acc[RB][CB];

// Position L of the grouped raster -> output tile (tm = weight-row tile, tn = token tile).  The token tiles
// are taken in super-blocks of tn_super tiles (the last one holds the rest; tn_super >= n_tn: one block):
// the grouped raster sweeps the token tiles of a block once per group of weight-row tiles, so the block's
// rows of the token operand are re-read once per group, and a block is sized to stay in the Infinity Cache
// between two sweeps.
__device__ __forceinline__ void tile_at(int L, int n_tm, int n_tn, int tn_super, int& tm, int& tn) {
  const int per_super = n_tm * tn_super;
  const int sb = L / per_super;
  const int tn0 = sb * tn_super;
  const int nt = min(tn_super, n_tn - tn0);
  const int in_sb = L - sb * per_super;
  const int per_group = kGroupM * nt;
  const int g = in_sb / per_group, in_g = in_sb - g * per_group;
  const int first_m = g * kGroupM;
  const int gsize = min(n_tm - first_m, kGroupM);
  tm = first_m + in_g % gsize;
  tn = tn0 + in_g / gsize;
}

// A copy of x the optimiser cannot see through.  Per-tile code derives its lane-dependent
// addressing from such a copy so that those values are recomputed per tile instead of being
// hoisted out of the tile loop, where they would occupy registers throughout the K loop.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Per-lane addressing of the operand stream.  Load j (0..3) of a wave fills the 1 KiB block
// (wave*4 + j) of an operand tile: 8 rows x 128 B.  Lane i lands at byte 16*i of the block, i.e. row i/8,
// physical chunk i%8, which holds logical chunk (i%8) ^ ((row>>1)&7).  Rows past the end of a matrix are
// clamped to its last row (their results are never stored); the buffer resources bound every access to
// the matrix anyway.
//
// The stream is a sequence of runs of K tiles.  Within a run the per-lane offsets stay put and the two
// scalar offsets advance by a fixed step per K tile.  A plain output tile is one run over the K tiles of
// its two matrices.  With side state (kSide) a tile's runs are: one per direction K tile, one over its
// bank K tiles, then the base run (see SideOperands).
struct OperandStream {
  __amdgpu_buffer_rsrc_t rA, rB;
  uint32_t offA[kLPW], offB[kLPW];
  int soffA, soffB;     // scalar byte offsets of the run's first K tile
  int stepA, stepB;     // their increments per K tile within the run
  int kt, len;          // the cursor's K tile within the run, K tiles of the run
  int L;                // raster position of the cursor's output tile
  int dir_next;         // kSide: direction K tiles of the tile already started
  int phase;            // kSide: 0 direction runs, 1 the bank run is under way, 2 the base run is
};

// Side operands of the probe GEMM as extra K tiles in front of the base K tiles (Sec. 3.2: the candidate
// term s eps (X V_k) U_k^T and the bank term (X Vb) P^T as LoRA-style factors).  Token side: pool K tile p
// is [256 tokens][64 columns] bf16; weight side: Uimg block e is [m_img][32] (one 32-column block of one
// direction's U), Pimg block b is [m_img][64].  Direction K tile j of a token tile multiplies the slots 2j
// and 2j+1 of the tile's slot list (columns 0-31 and 32-63 of the K tile); a token row is non-zero only
// in the slots of its own direction, and a foreground row is zero throughout, so its accumulators are
// still +0 when the base run starts: the state of a plain GEMM.
struct SideOperands {
  const TileHdr* hdr;
  const int32_t* slots;
  const bf16_t* Uimg; const bf16_t* Pimg; const bf16_t* Xs;
  int m_img;
  int uimg_bytes, pimg_bytes, xs_bytes;
};

// Rows of B that a lane's kLPW loads of a tile cover, when B's rows are gathered through a list
// (b_rows[j] = row of B behind position j; positions past n_b - 1 repeat the last one).
__device__ __forceinline__ void gather_rows(int (&idx)[kLPW], const int32_t* b_rows, int n_b, int tile_n0, int wave,
                                            int lane) {
#pragma unroll
  for (int j = 0; j < kLPW; ++j) idx[j] = b_rows[min(tile_n0 + (wave * kLPW + j) * 8 + (lane >> 3), n_b - 1)];
}

// The base run of an output tile.  B_rows_total: rows of the matrix B (only used with a gather list: the
// whole matrix is the buffer then).
template <bool kGather>
__device__ __forceinline__ void setup_stream(OperandStream& o, const bf16_t* A, int64_t lda, int M, int tile_m0,
                                             const bf16_t* B, int64_t ldb, int N, int tile_n0, int K, int wave,
                                             int lane, const int (&idx)[kLPW], int B_rows_total, bool half = false) {
  // (half: the A side of a half tile is 128 rows, two loads per wave: load j covers rows (2 wave + j) * 8 ...)
#pragma unroll
  for (int j = 0; j < kLPW; ++j) {
    const int row = (wave * kLPW + j) * 8 + (lane >> 3);
    const int lch = (lane & 7) ^ ((row >> 1) & 7);
    const int rowA = half ? (wave * 2 + (j & 1)) * 8 + (lane >> 3) : row;
    const int lchA = (lane & 7) ^ ((rowA >> 1) & 7);
    const int ra = min(tile_m0 + rowA, M - 1) - tile_m0;
    const int rbn = kGather ? idx[j] : min(tile_n0 + row, N - 1) - tile_n0;
    // 24-bit multiply: fewer than 2^24 rows, and the launchers reject row pitches of 16 MiB or more
    o.offA[j] = __umul24((uint32_t)ra, (uint32_t)lda * 2u) + lchA * 16;
    o.offB[j] = __umul24((uint32_t)rbn, (uint32_t)ldb * 2u) + lch * 16;
  }
  const int64_t bytesA = ((int64_t)(M - tile_m0 - 1) * lda + K) * 2;
  const int64_t bytesB = kGather ? ((int64_t)(B_rows_total - 1) * ldb + K) * 2 : ((int64_t)(N - tile_n0 - 1) * ldb + K) * 2;
  o.rA = __builtin_amdgcn_make_buffer_rsrc((void*)(A + (int64_t)tile_m0 * lda), 0,
                                           (int)min(bytesA, (int64_t)0x7FFFFFFF), 0x00020000);
  o.rB = __builtin_amdgcn_make_buffer_rsrc((void*)(kGather ? B : B + (int64_t)tile_n0 * ldb), 0,
                                           (int)min(bytesB, (int64_t)0x7FFFFFFF), 0x00020000);
  o.soffA = o.soffB = 0;
  o.stepA = o.stepB = BK * 2;
  o.kt = 0;
  o.len = K / BK;
  o.phase = 2;
}

// Per-lane offsets of a side run.  The images hold every row of a tile (they are padded), so a lane's
// offset is its row in the tile times the image's row pitch plus its swizzled chunk.
template <bool kDirRun>
__device__ __forceinline__ void setup_side_offsets(OperandStream& o, int wave, int lane, int base0, int base1, bool half) {
#pragma unroll
  for (int j = 0; j < kLPW; ++j) {
    const int row = (wave * kLPW + j) * 8 + (lane >> 3);
    const int lch = (lane & 7) ^ ((row >> 1) & 7);
    const int rowA = half ? (wave * 2 + (j & 1)) * 8 + (lane >> 3) : row;   // (as in setup_stream)
    const int lchA = (lane & 7) ^ ((rowA >> 1) & 7);
    o.offB[j] = row * 128 + lch * 16;
    // direction run: columns 0-31 of the K tile come from image block base0, columns 32-63 from base1
    o.offA[j] = kDirRun ? (uint32_t)((lchA >= 4 ? base1 : base0) + rowA * 64 + (lchA & 3) * 16) : (uint32_t)(rowA * 128 + lchA * 16);
  }
}

// Persistent GEMM driver.  For every output tile of this workgroup:
//   acc[rb][cb] = sum over the tile's K tiles (side K tiles first, then the K / 64 base K tiles) of
//                 A[tile rows] * B[tile rows]^T, starting from +0,
//   post(m0, n0, acc, row blocks per wave)  consumes the accumulators (it may use lds + kStagesLds .. +kEpiLds
//                      and workgroup barriers; it must not touch the operand stages).
// 16x16x32 fragments: lane l holds row l%16 and the 8 k-values of group l/16; D: lane l holds
// rows 4*(l/16) + v (v = 0..3) of column l%16.
//
// Pipeline of the K loop.  K tiles of 64 (128-byte row segments, so every L2 request is a
// full line) alternate between two LDS stages.  A K tile is two k-steps of 32; the 12 LDS
// reads of the next k-step's fragments are spread under the 32 MFMAs of the current one
// (an A fragment's registers are reused once its four MFMAs have issued).  The single
// barrier of a K tile sits between its two k-steps: by then every wave has read its last
// fragments of this K tile's stage (so the stage can be refilled) and the next K tile has
// landed (so its first fragments can be fetched under the second k-step).  The load cursor
// runs ahead of the compute cursor across runs and output-tile boundaries; past the
// workgroup's last tile it stays on the final K tile (those loads refill stages nobody
// reads again).  The K loop itself does not know what a K tile holds: side K tiles reach
// the matrix core through the same LDS stages as the base K tiles.
//
// With kGather the N rows of the B operand are rows b_rows[0..N-1] of a matrix of B_rows_total rows
// (smaller than 2 GiB); the row list of a tile is fetched one tile ahead of the load cursor.
template <bool kGather, bool kSplit, bool kSide, class Post>
__device__ __forceinline__ void persistent_gemm(const bf16_t* __restrict__ A, int64_t lda, int M,
                                                const bf16_t* __restrict__ B, int64_t ldb, int N, int K,
                                                int n_tm, int n_tn, int tn_super, int n_split, char* lds, Post post,
                                                const SideOperands& so,
                                                const int32_t* __restrict__ b_rows = nullptr, int B_rows_total = 0) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 2, wn = wave & 3;

  // Workgroup -> work items.  Consecutive workgroup ids land on consecutive XCDs, so blockIdx.x % 8
  // is the XCD and blockIdx.x / 8 a slot on it.  The raster is cut into chunks of `slots`
  // positions (32 on a full chip: an 8x4 block of tiles, 12 operand slices for 32 tiles in
  // that XCD's L2); chunk c goes to XCD c % 8, so at any time the eight XCDs work on eight
  // neighbouring chunks, which share their eight weight-row tiles: the weight slices reach
  // the chip once per step, not once per XCD.
  //
  // With kSplit the last n_split raster positions are two work items each, the halves of 128 A rows
  // of the tile: a last round that would occupy at most half of the workgroups with whole tiles
  // occupies twice as many with halves.  A half is a tile whose A rows start 128 further down and of
  // which only the first 128 A rows exist: the two wave rows take 64 of them each (4 instead of 8 row
  // blocks per wave), so every SIMD still has its two waves feeding the matrix core.  A workgroup has at
  // most one half and takes it last, on a pipeline of its own (three smaller stages; see below).
  // The K order of an output element is the same either way.
  const int total = n_tm * n_tn;
  const int first_split = total - (kSplit ? n_split : 0);
  const int xcd = blockIdx.x % kXcds;
  const int slots = gridDim.x / kXcds;
  const int stride = kXcds * slots;
  const int L_end = total + (kSplit ? n_split : 0);
  int L = xcd * slots + blockIdx.x / kXcds;
  if (L >= L_end) return;
  // item -> first A row, first B row of its tile; returns whether it is a half
  auto item_at = [&](int I, int& m0, int& n0) -> bool {
    int pos = I, half = 0;
    const bool is_half = kSplit && I >= first_split;
    if (is_half) {
      pos = first_split + ((I - first_split) >> 1);
      half = (I - first_split) & 1;
    }
    int tm, tn;
    tile_at(pos, n_tm, n_tn, tn_super, tm, tn);
    // (the integer divisions of the raster run on the vector ALU; their results are wave-uniform, and
    // saying so keeps everything derived from them in scalar registers)
    m0 = __builtin_amdgcn_readfirstlane(tm * BM + half * (BM / 2));
    n0 = __builtin_amdgcn_readfirstlane(tn * BN);
    return is_half;
  };
  const int nk = K / BK;
  // the side K tiles of the token tile that starts at row n0
  auto side_hdr = [&](int n0) -> TileHdr {
    TileHdr h = so.hdr[n0 / BN];
    h.kt0 = __builtin_amdgcn_readfirstlane(h.kt0);
    h.n_slots = __builtin_amdgcn_readfirstlane(h.n_slots);
    h.n_bank_kt = __builtin_amdgcn_readfirstlane(h.n_bank_kt);
    h.slot0 = __builtin_amdgcn_readfirstlane(h.slot0);
    return h;
  };

  // LDS -> register mapping
  const int r16 = lane & 15;
  const int swz = (r16 >> 1) & 7;
  uint32_t roff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) roff[ks] = r16 * 128 + (((ks * 4 + (lane >> 4)) ^ swz) << 4);
  const uint32_t aBaseWhole = wm * 128 * 128, aBaseHalf = wm * 64 * 128, bBase = kOperandStage + wn * 64 * 128;

  // load cursor.  It does not run past cursor_end: the whole tiles of the workgroup first, then (kSplit) its half.
  int cursor_end = first_split;
  OperandStream ld;
  int idx_next[kLPW] = {};   // gather: B rows of the tile after the cursor's
  // the next run of the cursor's output tile (the first one after ld.dir_next = 0, ld.phase = 0)
  auto next_run = [&]() {
    int m0, n0;
    const bool half = item_at(ld.L, m0, n0);
    if constexpr (kSide) {
      const TileHdr h = side_hdr(n0);
      const int n_dir_kt = (h.n_slots + 1) >> 1;
      const int lane_t = opaque(lane);
      if (ld.dir_next < n_dir_kt) {
        // direction K tile j: slots 2j and 2j+1 (an odd count leaves the second half of the last tile
        // to the first slot's block again; the token side holds zeros there)
        const int j = ld.dir_next;
        const int e0 = __builtin_amdgcn_readfirstlane(so.slots[h.slot0 + 2 * j]);
        const int e1 = 2 * j + 1 < h.n_slots ? __builtin_amdgcn_readfirstlane(so.slots[h.slot0 + 2 * j + 1]) : e0;
        setup_side_offsets<true>(ld, wave, lane_t, e0 * so.m_img * 64, e1 * so.m_img * 64, half);
        ld.rA = __builtin_amdgcn_make_buffer_rsrc((void*)so.Uimg, 0, so.uimg_bytes, 0x00020000);
        ld.rB = __builtin_amdgcn_make_buffer_rsrc((void*)so.Xs, 0, so.xs_bytes, 0x00020000);
        ld.soffA = m0 * 64;
        ld.soffB = (h.kt0 + j) * (BN * BK * 2);
        ld.stepA = ld.stepB = 0;
        ld.kt = 0;
        ld.len = 1;
        ld.dir_next = j + 1;
        return;
      }
      if (ld.phase == 0 && h.n_bank_kt > 0) {
        setup_side_offsets<false>(ld, wave, lane_t, 0, 0, half);
        ld.rA = __builtin_amdgcn_make_buffer_rsrc((void*)so.Pimg, 0, so.pimg_bytes, 0x00020000);
        ld.rB = __builtin_amdgcn_make_buffer_rsrc((void*)so.Xs, 0, so.xs_bytes, 0x00020000);
        ld.soffA = m0 * 128;
        ld.soffB = (h.kt0 + n_dir_kt) * (BN * BK * 2);
        ld.stepA = so.m_img * 128;
        ld.stepB = BN * BK * 2;
        ld.kt = 0;
        ld.len = h.n_bank_kt;
        ld.phase = 1;
        return;
      }
    }
    setup_stream<kGather>(ld, A, lda, M, m0, B, ldb, N, n0, K, wave, opaque(lane), idx_next, B_rows_total, half);
    if (kGather) {
      item_at(min(ld.L + stride, cursor_end - 1), m0, n0);
      gather_rows(idx_next, b_rows, N, n0, wave, lane);
    }
  };
  // (every scalar of the cursor is defined on every path: an undefined one would be given a vector register)
  ld.soffA = ld.soffB = ld.stepA = ld.stepB = ld.kt = ld.len = 0;
  auto start_cursor = [&](int at) {
    ld.L = at;
    ld.dir_next = 0;
    ld.phase = 0;
    if (kGather) {
      int m0, n0;
      item_at(at, m0, n0);
      gather_rows(idx_next, b_rows, N, n0, wave, lane);
    }
    next_run();
  };
  // load i (0..7) of the cursor's K tile: i < 4 -> A chunk i, else B chunk i - 4
  auto issue_range = [&](int stage, int first, int count) {
    char* sbase = lds + stage * kStage + wave * kLPW * 1024;
    int soffA = ld.soffA + ld.kt * ld.stepA, soffB = ld.soffB + ld.kt * ld.stepB;
    if constexpr (kSide) {
      // The cursor's scalars are wave-uniform, but with runs set up on several control-flow paths the
      // compiler keeps them in vector registers; a load whose scalar offset sits in a vector register is
      // wrapped in a lane-by-lane loop unless the offset is read back into a scalar register first.
      soffA = __builtin_amdgcn_readfirstlane(soffA);
      soffB = __builtin_amdgcn_readfirstlane(soffB);
    }
#pragma unroll
    for (int i = first; i < first + count; ++i) {
      if (i < kLPW)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rA, (lds_void*)(sbase + i * 1024), 16, (int)ld.offA[i], soffA, 0, 0);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rB, (lds_void*)(sbase + kOperandStage + (i - kLPW) * 1024), 16,
                                                 (int)ld.offB[i - kLPW], soffB, 0, 0);
    }
  };
  auto advance_cursor = [&]() {
    if (ld.kt + 1 < ld.len) {
      ++ld.kt;
      return;
    }
    if (!kSide || ld.phase == 2) {   // the tile's last K tile: on to the next output tile, if there is one
      if (ld.L + stride >= cursor_end) return;
      ld.L += stride;
      ld.dir_next = 0;
      ld.phase = 0;
    }
    next_run();
  };

  bf16x8 fa[2][RB], fb[2][CB];
  // token fragments first: every MFMA of the next k-step needs one of them
  auto load_frags = [&](int set, int stage, int ks, auto rb_c) {
    constexpr int kRB = decltype(rb_c)::value;   // row blocks of this wave: 8 in a whole tile, 4 in a half
    const char* s = lds + stage * kStage;
    const uint32_t aBase = kRB == RB ? aBaseWhole : aBaseHalf;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) fb[set][cb] = *(const bf16x8*)(s + bBase + cb * 2048 + roff[ks]);
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) fa[set][rb] = *(const bf16x8*)(s + aBase + rb * 2048 + roff[ks]);
  };
  // scheduling of one k-step with n_loads direct-to-LDS loads: in every group of 8 MFMAs,
  // 3 LDS reads (4 in a half, which has 8 reads for 16 MFMAs) and the loads spread evenly
  auto pattern = [&](auto n_loads_c, auto rb_c) {
    constexpr int n_loads = decltype(n_loads_c)::value;
    constexpr int kRB = decltype(rb_c)::value;
#pragma unroll
    for (int i = 0; i < kRB * CB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
      const int j = i & 7;
      if (kRB == RB ? (j == 0 || j == 3 || j == 5) : (j & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
      if (n_loads * (i + 1) / (kRB * CB) != n_loads * i / (kRB * CB))
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // direct-to-LDS load
    }
  };

  if (L < first_split) {
  start_cursor(L);
  // prologue: first K tile of the first output tile, and the late part of the second K tile's loads
  issue_range(0, 0, 2 * kLPW);
  advance_cursor();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  block_barrier();
  load_frags(0, 0, 0, std::integral_constant<int, RB>{});
  issue_range(1, 0, kLoadsLate);

  int stage = 0;
  for (; L < first_split; L += stride) {
    int m0, n0;
    item_at(L, m0, n0);
    int nk_tile = nk;
    if constexpr (kSide) {
      const TileHdr h = side_hdr(n0);
      nk_tile += ((h.n_slots + 1) >> 1) + h.n_bank_kt;
    }
    Acc acc;   // started by the first k-step's products
    // first_c: the tile's very first k-step, whose products start the accumulators (C = +0 as an operand,
    // so the accumulators need no clearing between tiles)
    auto mfmas = [&](int set, auto first_c) __attribute__((always_inline)) {
      constexpr bool kFirst = decltype(first_c)::value;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[set][rb], fb[set][cb],
                                                                 kFirst ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[rb][cb], 0, 0, 0);
    };
    constexpr std::integral_constant<int, RB> rb_c{};
    auto k_tile = [&](auto first_c) __attribute__((always_inline)) {
      // k-step 0: the rest of the next K tile's loads, fragments of k-step 1
      __builtin_amdgcn_sched_barrier(0);
      issue_range(stage ^ 1, kLoadsLate, kLoadsEarly);
      load_frags(1, stage, 1, rb_c);
      mfmas(0, first_c);
      pattern(std::integral_constant<int, kLoadsEarly>{}, rb_c);
      __builtin_amdgcn_sched_barrier(0);
      // the next K tile has landed; every wave is done reading this K tile's stage
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      block_barrier();
      advance_cursor();
      __builtin_amdgcn_sched_barrier(0);
      // k-step 1: first fragments of the next K tile, first loads of the one after it
      issue_range(stage, 0, kLoadsLate);
      load_frags(0, stage ^ 1, 0, rb_c);
      mfmas(1, std::false_type{});
      pattern(std::integral_constant<int, kLoadsLate>{}, rb_c);
      __builtin_amdgcn_sched_barrier(0);
      stage ^= 1;
    };
    // The first fragments of this tile were already fetched under the previous tile's last
    // k-step; fetching them again here keeps their registers free during post().
    load_frags(0, stage, 0, rb_c);
    k_tile(std::true_type{});   // (a tile has at least one K tile)
    for (int kt = 1; kt < nk_tile; ++kt) k_tile(std::false_type{});
    post(m0, n0, acc, rb_c);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the trailing loads
  }

  // The workgroup's half tile, if it has one (at most one: the halves are the last 2 n_split <= gridDim.x work
  // items, and it is the workgroup's last item).  With half the products per K tile, a K tile's period would
  // meet the latency of loads requested one period ahead; a half needs only 48 KiB per stage, so it runs on
  // three stages with every K tile requested two periods ahead.
  if constexpr (kSplit) {
    if (L < L_end) {
      constexpr std::integral_constant<int, RB / 2> rb_c{};
      constexpr int kHalfLoads = 2 + kLPW;   // loads of a wave per K tile: 2 of the 128 A rows, 4 of the 256 B rows
      block_barrier();   // the whole tiles' stages and epilogue scratch are free: every wave is past them
      cursor_end = L_end;
      start_cursor(L);
      int m0, n0;
      item_at(L, m0, n0);
      int nk_tile = nk;
      if constexpr (kSide) {
        const TileHdr h = side_hdr(n0);
        nk_tile += ((h.n_slots + 1) >> 1) + h.n_bank_kt;
      }
      auto issue_half = [&](int stg) {
        char* sb = lds + stg * kHalfStage;
        int soffA = ld.soffA + ld.kt * ld.stepA, soffB = ld.soffB + ld.kt * ld.stepB;
        if constexpr (kSide) {
          soffA = __builtin_amdgcn_readfirstlane(soffA);
          soffB = __builtin_amdgcn_readfirstlane(soffB);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rA, (lds_void*)(sb + (wave * 2 + j) * 1024), 16, (int)ld.offA[j], soffA, 0, 0);
#pragma unroll
        for (int j = 0; j < kLPW; ++j)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rB, (lds_void*)(sb + kHalfA + (wave * kLPW + j) * 1024), 16,
                                                   (int)ld.offB[j], soffB, 0, 0);
      };
      auto frags_half = [&](int set, int stg, int ks) {
        const char* sb = lds + stg * kHalfStage;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) fb[set][cb] = *(const bf16x8*)(sb + kHalfA + wn * 64 * 128 + cb * 2048 + roff[ks]);
#pragma unroll
        for (int rb = 0; rb < RB / 2; ++rb) fa[set][rb] = *(const bf16x8*)(sb + wm * 64 * 128 + rb * 2048 + roff[ks]);
      };
      Acc acc;
      auto mfmas = [&](int set, auto first_c) __attribute__((always_inline)) {
        constexpr bool kFirst = decltype(first_c)::value;
#pragma unroll
        for (int rb = 0; rb < RB / 2; ++rb)
#pragma unroll
          for (int cb = 0; cb < CB; ++cb)
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[set][rb], fb[set][cb],
                                                                   kFirst ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[rb][cb], 0, 0, 0);
      };
      // K tiles 0, 1, 2 into the three stages (past the item's last K tile the cursor stays on it)
      issue_half(0);
      advance_cursor();
      issue_half(1);
      advance_cursor();
      issue_half(2);
      asm volatile("s_waitcnt vmcnt(12)" ::: "memory");   // K tile 0 has landed (2 x 6 loads may be outstanding)
      static_assert(kHalfLoads == 6, "the counts of the waits above and below");
      block_barrier();
      frags_half(0, 0, 0);
      int stg = 0;
      auto k_tile = [&](auto first_c) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        frags_half(1, stg, 1);
        mfmas(0, first_c);
        pattern(std::integral_constant<int, 0>{}, rb_c);
        __builtin_amdgcn_sched_barrier(0);
        // the next K tile has landed (only the six loads of the one after it may be outstanding); every wave is
        // done reading this K tile's stage, which takes the K tile three ahead
        asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)" ::: "memory");
        block_barrier();
        advance_cursor();
        __builtin_amdgcn_sched_barrier(0);
        issue_half(stg);
        const int nxt = stg == 2 ? 0 : stg + 1;
        frags_half(0, nxt, 0);
        mfmas(1, std::false_type{});
        pattern(std::integral_constant<int, kHalfLoads>{}, rb_c);
        __builtin_amdgcn_sched_barrier(0);
        stg = nxt;
      };
      k_tile(std::true_type{});
      for (int kt = 1; kt < nk_tile; ++kt) k_tile(std::false_type{});
      post(m0, n0, acc, rb_c);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the trailing loads before the workgroup ends
    }
  }
}

// Compute units of the current device, cached per device.
int compute_units() {
  static std::atomic<int> cus[kMaxDevices];
  const int dev = current_device();
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < kXcds) n = 256;
    cus[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// How many of the last tiles of the raster are cut into two halves of 128 weight rows: all tiles of a last
// round that would leave at least half of the workgroups without one.  Only when every tile has rows in
// both halves (the last weight-row tile holds more than 128 rows), so that no half is empty.
static int split_tiles(int total_tiles, int m) {
  const int cus = compute_units();
  const int rem = total_tiles % cus;
  if (rem == 0 || rem > cus / 2 || (m - 1) % BM < BM / 2) return 0;
  return rem;
}

// Token tiles per super-block of the raster.  Every group of 8 weight-row tiles sweeps all token tiles of a
// block; a token operand beyond what the 256 MB Infinity Cache keeps between two sweeps is cut into blocks
// of at most 128 MB of rows (a multiple of the 4 token tiles of an XCD's block).  The weight matrix is then
// streamed once per block instead of once.
static int token_super_block(int n_tn, int64_t token_operand_bytes) {
  if (token_operand_bytes <= (192ll << 20)) return n_tn;
  const int n_super = (int)((token_operand_bytes + (128ll << 20) - 1) / (128ll << 20));
  return ((n_tn + n_super - 1) / n_super + 3) / 4 * 4;
}

static int gemm_grid(int total_tiles) {
  const int cus = compute_units();
  const int per_xcd = (total_tiles + kXcds - 1) / kXcds;
  const int slots = per_xcd < cus / kXcds ? per_xcd : cus / kXcds;
  return slots * kXcds;
}

// ---------------------------------------------------------------------------------------
// Probe linear.  Side K tiles first, base K tiles second: the accumulators of a foreground
// token are still +0 when the base K tiles start (its side operand rows are zero), i.e.
// exactly the state a plain GEMM starts from, so foreground rows come out bit-identical
// to an all-foreground call.
// ---------------------------------------------------------------------------------------
// 16-byte store of finished outputs with the non-temporal hint: a tile's 128 KiB of Y are written once
// and read by a later kernel at the earliest, so they should not displace operand slices from the
// caches (measured on the 20480 x 5120 layer at 16384 rows: 2.64 -> 2.58 ms; with no stores at all 2.56).
__device__ __forceinline__ void store_streaming(bf16_t* dst, u32x4 val) {
  __builtin_nontemporal_store(val, (u32x4*)dst);
}

// silu(gate) * up, the gated-MLP epilogue (activation 2): adjacent output features are (gate, up) pairs
__device__ __forceinline__ float silu_mul(float gate, float up) { return gate / (1.0f + __expf(-gate)) * up; }

// kSplit: the variant whose last round is made of half tiles (n_split > 0); the launcher takes it only when
// the tile count leaves such a round, so every other shape runs the loop without the extra branches.
template <bool kSide, bool kOutBf16, bool kBias, bool kGate, bool kSplit>
__global__ __launch_bounds__(kThreads, 1) void k_probe_gemm(ProbeGemmArgs p, int n_tm, int n_tn, int tn_super, int n_split) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 2, wn = wave & 3;

  // D block (rb, cb): out feature = obase + rb*16 + 4*g + v, token = tbase + cb*16 + r16.  kRB = row blocks of
  // this wave: 8 (128 out features) in a whole tile, 4 (64) in a half.
  auto epilogue = [&](int tile_o0, int tile_t0, Acc& acc, auto rb_c) {
    constexpr int kRB = decltype(rb_c)::value;
    const int lane_t = opaque(lane);
    const int r16 = lane_t & 15, g = lane_t >> 4;
    const int obase = tile_o0 + wm * (kRB * 16);   // first out feature of this wave
    const int tbase = tile_t0 + wn * 64;           // first token of this wave
    // ReLU as a select on the sign, which lets a NaN through (a max would replace it by the other operand)
    const bool relu = p.act == 1;
    if constexpr (!kOutBf16) {
      float* Y = (float*)p.Y;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        const int t = tbase + cb * 16 + r16;
        if (t >= p.T) continue;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
          const int o0 = obase + rb * 16 + 4 * g;   // this lane's 4 consecutive out features
          float y[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            y[v] = acc[rb][cb][v];
            if constexpr (kBias) y[v] += p.bias[min(o0 + v, p.m - 1)];
          }
          if constexpr (kGate) {   // m is even, so a pair is inside or outside as a whole
            if (o0 < p.m) Y[(int64_t)t * p.ldy + (o0 >> 1)] = silu_mul(y[0], y[1]);
            if (o0 + 2 < p.m) Y[(int64_t)t * p.ldy + (o0 >> 1) + 1] = silu_mul(y[2], y[3]);
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (o0 + v < p.m) Y[(int64_t)t * p.ldy + o0 + v] = (relu && y[v] < 0.0f) ? 0.0f : y[v];
          }
        }
      }
      return;
    }
    if constexpr (kGate) {
      // bf16, gated: a lane's 4 features become 2 outputs (one dword); 16 tokens x (kRB * 8) outputs at a time
      // through this wave's LDS region (16-byte slots XOR-swizzled by the token), then 16-byte stores
      // covering kRB * 16 contiguous bytes per token row.
      constexpr int CH = kRB;                   // 16-byte chunks of a token row
      char* region = kRB == RB ? lds + kStagesLds + wave * 4096 : lds + kHalfStagesLds + wave * 2048;
      bf16_t* Y = (bf16_t*)p.Y;
      const int chunk = lane_t & (CH - 1);      // 8 outputs (16 bytes) of a token row
      const int oo = (obase >> 1) + chunk * 8;  // first of them
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = acc[rb][cb][e];
          if constexpr (kBias) {
            const int ob = obase + rb * 16 + 4 * g;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] += p.bias[min(ob + e, p.m - 1)];
          }
          // outputs rb*8 + 2g, +1 of the token's kRB*8: slot rb, bytes 4g..4g+3
          *(uint32_t*)(region + r16 * (CH * 16) + ((rb ^ (r16 & (CH - 1))) << 4) + 4 * g) =
              pack_bf16x2(silu_mul(y[0], y[1]), silu_mul(y[2], y[3]));
        }
        // the wave reads back what it wrote itself: LDS operations of one wave complete in order
#pragma unroll
        for (int it = 0; it < CH / 4; ++it) {
          const int tl = it * (64 / CH) + lane_t / CH;
          const int t = tbase + cb * 16 + tl;
          const u32x4 val = *(const u32x4_alias*)(region + tl * (CH * 16) + ((chunk ^ (tl & (CH - 1))) << 4));
          if (t < p.T && oo < (p.m >> 1)) store_streaming(Y + (int64_t)t * p.ldy + oo, val);   // m % 16 == 0
        }
      }
      return;
    }
    // bf16: bias / activation / rounding in registers, then 16 tokens x (kRB * 16) features at a
    // time through this wave's own 4 KiB of LDS (XOR-swizzled 16-byte slots) so that the
    // global stores are 16 bytes per lane and cover kRB * 32 contiguous bytes per token row.
    constexpr int CH = kRB * 2;                 // 16-byte chunks of a token row
    char* region = kRB == RB ? lds + kStagesLds + wave * 4096 : lds + kHalfStagesLds + wave * 2048;   // (a half: 2 KiB)
    bf16_t* Y = (bf16_t*)p.Y;
    const int chunk = lane_t & (CH - 1);        // 8 out features (16 bytes) of a token row
    const int o = obase + chunk * 8;
    const uint32_t wr_base = r16 * (CH * 16) + (g & 1) * 8;
    const uint32_t wr_swz = (r16 & (CH - 1)) * 16;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) {
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = acc[rb][cb][e];
        if constexpr (kBias) {
          const int ob = obase + rb * 16 + 4 * g;   // this lane's 4 consecutive out features
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] += p.bias[min(ob + e, p.m - 1)];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (relu && y[e] < 0.0f) ? 0.0f : y[e];
        // 16-byte slot rb*2 + g/2 of the token's row, half g&1
        *(u32x2_alias*)(region + wr_base + (((rb * 2 + (g >> 1)) * 16) ^ wr_swz)) =
            u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
      }
      // the wave reads back what it wrote itself: LDS operations of one wave complete in order
#pragma unroll
      for (int it = 0; it < CH / 4; ++it) {
        const int tl = it * (64 / CH) + lane_t / CH;
        const int t = tbase + cb * 16 + tl;
        const u32x4 val = *(const u32x4_alias*)(region + tl * (CH * 16) + ((chunk ^ (tl & (CH - 1))) * 16));
        if (t < p.T && o < p.m) store_streaming(Y + (int64_t)t * p.ldy + o, val);   // m % 8 == 0
      }
    }
  };

  SideOperands so;
  so.hdr = p.tile_hdr; so.slots = p.tile_slots; so.Uimg = p.Uimg; so.Pimg = p.Pimg; so.Xs = p.Xs; so.m_img = p.m_img;
  so.uimg_bytes = (int)p.uimg_bytes; so.pimg_bytes = (int)p.pimg_bytes; so.xs_bytes = (int)p.xs_bytes;
  persistent_gemm<false, kSplit, kSide>(p.W, p.ldw, p.m, p.X, p.ldx, p.T, p.n, n_tm, n_tn, tn_super, n_split, lds, epilogue, so);
}

template <bool kSide, bool kOutBf16, bool kBias, bool kGate, bool kSplit>
static hipError_t launch_probe_kernel(const ProbeGemmArgs& a, int n_tm, int n_tn, int n_split, hipStream_t st) {
  const int tn_super = token_super_block(n_tn, (int64_t)a.T * a.n * 2);
  static std::atomic<bool> configured[kMaxDevices];
  const hipError_t ec = once_per_device(configured, [] {
    return hipFuncSetAttribute((const void*)k_probe_gemm<kSide, kOutBf16, kBias, kGate, kSplit>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
  });
  if (ec != hipSuccess) return ec;
  hipLaunchKernelGGL((k_probe_gemm<kSide, kOutBf16, kBias, kGate, kSplit>), dim3(gemm_grid(n_tm * n_tn + n_split)),
                     dim3(kThreads), kGemmLds, st, a, n_tm, n_tn, tn_super, n_split);
  return hipGetLastError();
}

template <bool kSide, bool kOutBf16, bool kBias, bool kGate>
static hipError_t launch_probe_variant(const ProbeGemmArgs& a, hipStream_t st) {
  const int n_tm = (a.m + BM - 1) / BM, n_tn = (a.T + BN - 1) / BN;
  const int n_split = split_tiles(n_tm * n_tn, a.m);
  return n_split > 0 ? launch_probe_kernel<kSide, kOutBf16, kBias, kGate, true>(a, n_tm, n_tn, n_split, st)
                     : launch_probe_kernel<kSide, kOutBf16, kBias, kGate, false>(a, n_tm, n_tn, 0, st);
}

template <bool kSide, bool kOutBf16>
static hipError_t launch_probe_bias(const ProbeGemmArgs& a, hipStream_t st) {
  if (a.act == 2)
    return a.bias ? launch_probe_variant<kSide, kOutBf16, true, true>(a, st)
                  : launch_probe_variant<kSide, kOutBf16, false, true>(a, st);
  return a.bias ? launch_probe_variant<kSide, kOutBf16, true, false>(a, st)
                : launch_probe_variant<kSide, kOutBf16, false, false>(a, st);
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

// kGather: only the scored tokens (rows p.rows[0 .. *p.n_rows - 1] of H) are multiplied; token tiles
// and the partial outputs then run over positions in that list.
template <bool kGather>
__global__ __launch_bounds__(kThreads, 1) void k_head_score(HeadScoreArgs p, int n_tm, int tn_super) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int n_tok = kGather ? __builtin_amdgcn_readfirstlane(*p.n_rows) : p.T;   // tokens to score
  if (n_tok == 0) return;
  const int n_tn = (n_tok + BN - 1) / BN;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int wm = wave >> 2, wn = wave & 3;
  float* s_max = (float*)(lds + kStagesLds);   // [2 wave rows][256 tokens]
  float* s_sum = s_max + 2 * BN;                // [2 wave rows][256 tokens]
  constexpr float kLog2e = 1.4426950408889634f;

  // D block (rb, cb): vocabulary row = vbase + rb*16 + 4*g + v, token = tile_t0 + wn*64 + cb*16 + r16.
  auto epilogue = [&](int tile_v0, int tile_t0, Acc& acc, auto) {
    const int lane_t = opaque(lane), tid_t = opaque(tid);
    const int r16 = lane_t & 15, g = lane_t >> 4;
    const int tm = tile_v0 / BM;   // vocabulary tile: the index of this tile's partials
    const int vbase = tile_v0 + wm * 128;  // first vocabulary row of this wave
    if (tile_v0 + BM > p.vocab) {   // the last vocabulary tile: rows past the end count as -inf
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (vbase + rb * 16 + 4 * g + v >= p.vocab) acc[rb][cb][v] = -INFINITY;
    }
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const int tl = wn * 64 + cb * 16 + r16;   // token within the tile
      const int t = tile_t0 + tl;               // its position (in the list of scored tokens, or its row)
      float mx = -INFINITY;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) mx = fmaxf(mx, acc[rb][cb][v]);
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // sum of exp(z - max) as 2^(z log2(e) - max log2(e)), one multiply-add per logit
      const float mref2 = (mx == -INFINITY) ? 0.0f : -mx * kLog2e;
      float sum = 0.0f;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[rb][cb][v], kLog2e, mref2));
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      if (g == 0) { s_max[wm * BN + tl] = mx; s_sum[wm * BN + tl] = sum; }
      // target logit: exactly one lane of the whole grid holds it
      if (t < n_tok) {
        const int loc = p.targets[kGather ? p.rows[t] : t] - vbase;
        if (loc >= 0 && loc < 128 && ((loc >> 2) & 3) == g) {
          const int sel = (loc >> 4) * 4 + (loc & 3);
          float z = 0.0f;
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (sel == rb * 4 + v) z = acc[rb][cb][v];
          p.tgt_logit[t] = z;
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    block_barrier();   // (not __syncthreads: the operand loads of the next tile stay in flight)
    {
      const int t = tile_t0 + tid_t;
      if (tid_t < BN && t < n_tok) {
        const float m0 = s_max[tid_t], m1 = s_max[BN + tid_t];
        const float Mx = fmaxf(m0, m1);
        const float mref = (Mx == -INFINITY) ? 0.0f : Mx;
        const float S = s_sum[tid_t] * __builtin_amdgcn_exp2f((m0 - mref) * kLog2e) +
                        s_sum[BN + tid_t] * __builtin_amdgcn_exp2f((m1 - mref) * kLog2e);
        p.part_max[(int64_t)tm * p.T + t] = Mx;
        p.part_sum[(int64_t)tm * p.T + t] = S;
      }
    }
    // (no barrier here: the exchange buffers are written again after the next tile's K loop, whose barriers
    // every thread passes only after these reads)
  };

  persistent_gemm<kGather, false, false>(p.Wh, p.ldw, p.vocab, p.H, p.ldh, n_tok, p.d, n_tm, n_tn, tn_super, 0, lds, epilogue,
                                         SideOperands{}, p.rows, p.T);
}

template <bool kGather>
static hipError_t launch_head_variant(const HeadScoreArgs& a, hipStream_t st) {
  static std::atomic<bool> configured[kMaxDevices];
  const hipError_t ec = once_per_device(configured, [] {
    return hipFuncSetAttribute((const void*)k_head_score<kGather>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
  });
  if (ec != hipSuccess) return ec;
  // the grid is sized for every token being scored; with fewer, the surplus workgroups find no tile
  const int n_tm = (a.vocab + BM - 1) / BM, n_tn = (a.T + BN - 1) / BN;
  const int tn_super = token_super_block(n_tn, (int64_t)a.T * a.d * 2);
  hipLaunchKernelGGL(k_head_score<kGather>, dim3(gemm_grid(n_tm * n_tn)), dim3(kThreads), kGemmLds, st, a, n_tm, tn_super);
  return hipGetLastError();
}

hipError_t launch_head_score_bf16(const HeadScoreArgs& a, hipStream_t st) {
  if (a.T == 0) return hipSuccess;
  return a.rows ? launch_head_variant<true>(a, st) : launch_head_variant<false>(a, st);
}

}  // namespace zo
