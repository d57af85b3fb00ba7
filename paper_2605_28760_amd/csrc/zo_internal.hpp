// Internal interface between the host-side ABI (validation, workspace
// planning) and the kernel launchers.  Nothing here is exported.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace zo {

// Row-tile of the MFMA GEMM kernels and row-chunk of the side-down kernel.
constexpr int kTileM = 256;
constexpr int kTileN = 256;
constexpr int kTileK = 64;
constexpr int kMaxRank = 512;     // largest probe rank r (the rank continuum of Sec. 3.3 goes up to 512)
constexpr int kSideRows = 64;     // most rows of a side-down work item (one wave); small batches use 32 or 16
constexpr int kSideWaves = 8;    // waves (items) per workgroup of the side-down pass, at most
// LDS of a side-down workgroup of w waves whose items have rb 16-row blocks, next to nbb 16-column bank blocks:
// per wave two stages of its rows of X and one of its direction block of V, per workgroup two stages of Vb.
constexpr int side_lds_bytes(int nbb, int rb, int w) { return w * (2 * rb * 2048 + 2048) + 2 * (nbb > 0 ? nbb : 1) * 2048; }
// Waves (items) per workgroup: eight, or seven where eight would not fit the 160 KiB of a compute unit's LDS
// (64-row items next to eight bank blocks).
constexpr int side_waves_of(int nbb, int rb) { return side_lds_bytes(nbb, rb, kSideWaves) <= 160 * 1024 ? kSideWaves : kSideWaves - 1; }
constexpr int kSideMaxBlocks = 9; // 16-column blocks a side-down wave accumulates at once
constexpr int kSimtTile = 64;     // tile edge of the fp32 vector-ALU kernels

struct BatchDev {
  int T, S, C, K;
  const int32_t* cu;
  const int32_t* seq_cand;
  const int32_t* cand_dir;
  const float* cand_sign;
  const uint64_t* seed;
  const uint64_t* seed_v;   // null: V is drawn from `seed` too
};

// One side-down work item: rows [row0, row0 + nrows) of one sequence.
struct SideItem {
  int32_t row0;
  int32_t nrows;
  int32_t kind;   // direction index >= 0, kKindCentre or kKindForeground
  float scale;    // sign * eps
};

// Side K tiles of one token tile of the bf16 probe GEMM (a tile = kTileN packed rows).  The side state
// enters the GEMM as extra K tiles in front of the base K tiles: first the direction tiles (two slots
// of 32 columns each per K tile; a slot holds one 32-column block of one direction's U), then the bank
// tiles (64 bank columns each).
struct TileHdr {
  int32_t kt0;        // first K tile of this token tile in the pool of token-side images
  int32_t n_slots;    // direction slots in use (distinct directions of the tile x blocks per direction)
  int32_t n_bank_kt;  // bank K tiles (0 when the tile holds no candidate row)
  int32_t slot0;      // first entry of this tile in the slot list
};

struct SeqTables {
  int32_t* seq_kind;   // [S]
  float* seq_scale;    // [S]
  int32_t* tok_seq;    // [T]
  SideItem* items;     // [max_items]
  int32_t* n_items;    // [2]: number of side-down items, number of pool K tiles in use
  int32_t max_items;
  int32_t item_rows;   // rows per side-down item: 64, 48, 32 or 16
  // per token tile (null tile_hdr: not wanted)
  TileHdr* tile_hdr;   // [n_tn]
  int32_t* tile_slots; // [slot_cap]: block of the U image (direction * SPD + 32-column block) behind a slot
  int32_t* kt_tile;    // [kt_cap]: token tile that owns a pool K tile
  int32_t n_tn, slot_cap, kt_cap;
  int32_t SPD;         // 32-column blocks per direction
  int32_t RpT;         // bank K tiles of a tile with candidates
};

// number of compute units of the current device (256 on MI355X; cached per device)
int compute_units();

// Per-device, thread-safe one-time set-up of a kernel (its dynamic LDS limit).  `done` is a static
// array of the caller, one flag per device; the set-up call is idempotent, so two threads that race
// on the first launch both make it and both succeed.
constexpr int kMaxDevices = 64;
inline int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
  return dev;
}
template <class F>
inline hipError_t once_per_device(std::atomic<bool> (&done)[kMaxDevices], F setup) {
  const int dev = current_device();
  if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
  const hipError_t e = setup();
  if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
  return e;
}

// ---- zo_prep.hip ------------------------------------------------------------
hipError_t launch_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t first_block,
                               int64_t n_blocks, uint32_t* out, hipStream_t st);
hipError_t launch_factor_fill(uint64_t seed, uint32_t tensor_id, int64_t rows, int r, int bf16,
                              void* out, hipStream_t st);
hipError_t launch_tok_index(const BatchDev& b, int32_t* tok_seq, int32_t* tok_cand, hipStream_t st);
hipError_t launch_seq_tables(const BatchDev& b, float eps, const SeqTables& t, hipStream_t st);
// bf16 operand images.  For the GEMM's side K tiles: Uimg [K * SPD][m_img][32] (32-column blocks of U,
// 64-byte rows), Pimg [RpT][m_img][64] (64-column blocks of P, 128-byte rows); rows >= m and columns
// beyond the rank are zero.  For the side-down pass: Vt [K][RP][n] (V transposed), Vbt [Rp][n].
// fp32 factors: Uf [K][m][r], Vf [K][n][r]
hipError_t launch_factors_f32(const BatchDev& b, uint32_t tensor_id, int m, int n, int r,
                              float* Uf, float* Vf, hipStream_t st);

// ---- zo_side.hip --------------------------------------------------------------
struct SideDownArgs {
  const uint16_t* X; int64_t ldx;   // bf16 [T][n]
  const uint16_t* Vt;               // [K][RP][n]
  const uint16_t* Vbt;              // [Rp][n]
  int n, RP, Rp, T;
  const SideItem* items; const int32_t* n_items; int max_items;
  int item_rows;                    // rows per item: 64, 48, 32 or 16
  int ksplit;                       // >= 1: K ranges per row, a function of n alone (side_ksplit)
  float* partial;                   // [ksplit][T][RP+Rp] partial sums of one K range each
  const int32_t* tok_seq; const int32_t* seq_kind; const float* seq_scale;
  // where the finished rows go: the token-side images of the GEMM's side K tiles
  const TileHdr* tile_hdr; const int32_t* tile_slots; const int32_t* kt_tile;
  int kt_cap, SPD;
  uint16_t* Xs;                     // [pool K tile][kTileN][kTileK] bf16
};
// K ranges of the side-down pass for an input width n: never a function of the batch, so that the
// summation order of a row's side term does not depend on what else is in the batch.
int side_ksplit(int n);
// Rows per side-down work item (64, 48, 32 or 16) for a batch of T rows, input width n and bank rank R; how rows
// are grouped into items does not enter any row's arithmetic.
int side_item_rows(const int32_t* host_cu, const int32_t* host_seq_cand, int S, int T, int n, int R);
// sequence tables, token -> sequence map and the four operand images of a bf16 probe linear in one launch
hipError_t launch_probe_prep_bf16(const BatchDev& b, float eps, const SeqTables& tabs, uint32_t tensor_id, int m,
                                  int n, int r, int RP, int Rp, const float* P, const float* Vb, int R_cap,
                                  int R_used, int m_img, uint16_t* Uimg, uint16_t* Vt, uint16_t* Pimg, uint16_t* Vbt,
                                  hipStream_t st);
hipError_t launch_side_down_bf16(const SideDownArgs& a, hipStream_t st);

// ---- zo_gemm.hip ---------------------------------------------------------------
struct ProbeGemmArgs {
  const uint16_t* X; int64_t ldx;
  const uint16_t* W; int64_t ldw;
  const float* bias;
  int T, m, n;
  int act;
  void* Y; int64_t ldy; int out_bf16;
  // side state (has_side = 0: plain GEMM for every row): extra K tiles in front of the base K tiles
  int has_side;
  const TileHdr* tile_hdr;          // [token tiles]
  const int32_t* tile_slots;
  const uint16_t* Uimg;             // [K * SPD][m_img][32]
  const uint16_t* Pimg;             // [RpT][m_img][64]
  const uint16_t* Xs;               // [pool K tile][kTileN][kTileK]
  int m_img;                        // rows of the images: the weight-row tiles rounded up, plus half a tile
  int64_t uimg_bytes, pimg_bytes, xs_bytes;
};
hipError_t launch_probe_gemm_bf16(const ProbeGemmArgs& a, hipStream_t st);

struct HeadScoreArgs {
  const uint16_t* H; int64_t ldh;
  const uint16_t* Wh; int64_t ldw;
  int T, vocab, d;
  const int32_t* targets;
  float* part_max;                  // [n_vt][T]
  float* part_sum;                  // [n_vt][T]
  float* tgt_logit;                 // [T]
  // scored rows only (both null: every row of H is multiplied).  rows[j] = row of H of the j-th scored
  // token, *n_rows = their number; the partial outputs are then indexed by j instead of the row
  const int32_t* rows; const int32_t* n_rows;
};
int head_vocab_tiles_bf16(int vocab);
hipError_t launch_head_score_bf16(const HeadScoreArgs& a, hipStream_t st);

// ---- zo_simt.hip (fp32 on the vector ALU) ------------------------------------------
struct ProbeF32Args {
  const float* X; int64_t ldx;
  const float* W; int64_t ldw;
  const float* bias;
  int T, m, n, r, R, R_cap;
  int act;
  float* Y; int64_t ldy;
  int has_side;
  const int32_t* tok_seq; const int32_t* seq_kind; const float* seq_scale;
  const float* Uf; const float* Vf;  // [K][m][r], [K][n][r]
  const float* P; const float* Vb;   // bank, ld R_cap
  float* Tside;                      // [T][r+R]
};
hipError_t launch_probe_f32(const ProbeF32Args& a, hipStream_t st);
int head_vocab_tiles_f32(int vocab);
struct HeadScoreF32Args {
  const float* H; int64_t ldh;
  const float* Wh; int64_t ldw;
  int T, vocab, d;
  const int32_t* targets;
  float* part_max; float* part_sum; float* tgt_logit;
};
hipError_t launch_head_score_f32(const HeadScoreF32Args& a, hipStream_t st);

// ---- zo_reduce.hip -------------------------------------------------------------------
struct ScoreCombineArgs {
  int T, S, C, n_vt;
  const float* part_max; const float* part_sum; const float* tgt_logit;
  const int32_t* targets;
  const int32_t* pos;  // [T] index of a scored token in the partial arrays (null: the token's own row)
  const int32_t* cu; const int32_t* seq_cand;
  float* tok_nll;      // [T] (workspace when the caller passes none)
  float* seq_nll;      // [S]
  int32_t* seq_cnt;    // [S] workspace
  float* cand_sum;     // [C]
  int32_t* cand_cnt;   // [C]
};
hipError_t launch_score_combine(const ScoreCombineArgs& a, hipStream_t st);
// rows[j] = j-th token with targets >= 0 (ascending), pos[t] = number of such tokens before t, *n_rows = their count
hipError_t launch_active_rows(const int32_t* targets, int T, int32_t* rows, int32_t* pos, int32_t* n_rows, hipStream_t st);
hipError_t launch_estimate(const BatchDev& b, const float* cand_sum, const int32_t* cand_cnt, float eps,
                           int reduction, float* cand_loss, float* proj_grad, hipStream_t st);
// Device-resident schedule state (same layout as the zo_sched of the public header).
struct SchedDev {
  int64_t next_step, step;
  int32_t interval, block, append, reserved;
};
hipError_t launch_schedule_step(SchedDev* s, int nu, int n_blocks, int K, uint64_t base_u, uint64_t base_v,
                                uint64_t* seed_u, uint64_t* seed_v, hipStream_t st);

hipError_t launch_estimate_es(const BatchDev& b, const float* cand_sum, const int32_t* cand_cnt, float eps,
                              int reduction, float* cand_loss, float* proj_grad, hipStream_t st);
struct BankUpdateArgs {
  float* P; float* Vb; int R_cap;
  int m, n, r;
  const uint64_t* seed; const uint64_t* seed_v; uint32_t tensor_id;
  const SchedDev* sched; int n_dirs;   // sched non-null: block and mode come from the device
  const float* proj_grad; float lr; const float* dir_weight; float default_weight;
  int append; int bf16;
};
// col0: host array of n_dirs block offsets (passed to the kernel by value in batches)
hipError_t launch_bank_update(const BankUpdateArgs& a, int n_dirs, const int32_t* col0, hipStream_t st);
// the same update (same seeds, coefficients and column blocks) for many layers in one launch per 48 layers
struct BankLayer { float* P; float* Vb; int32_t R_cap, m, n; uint32_t tensor_id; };
constexpr int kBankMaxLayers = 48;
struct BankLayerSet { BankLayer l[kBankMaxLayers]; };
hipError_t launch_bank_update_multi(const BankUpdateArgs& common, const BankLayer* layers, int n_layers, int n_dirs,
                                    const int32_t* col0, hipStream_t st);

// W (fp32 or bf16, in place) += P[:, :R] Vb[:, :R]^T, then the R columns of P and Vb are zeroed.
struct FoldArgs {
  float* P; float* Vb; int R_cap, R;
  void* W; int64_t ldw; int m, n; int bf16;
};
hipError_t launch_fold_bank(const FoldArgs& a, hipStream_t st);

// ---- zo_block.hip (what joins the probe linears of a decoder block) --------------------
struct NormArgs {
  const void* X; int64_t ldx;       // [T][d]
  const void* R; int64_t ldr;       // optional residual added to X first
  const float* gamma; const float* beta;   // beta may be null
  int kind;                         // 0 layer norm, 1 RMS norm
  float eps;
  int T, d, bf16;
  void* Hsum; int64_t ldh;          // optional: X + R (may alias X)
  void* Y; int64_t ldy;             // optional: the normalised rows
};
hipError_t launch_add_norm(const NormArgs& a, hipStream_t st);

struct AttnArgs {
  const void* Q; int64_t ldq;       // [T][n_heads * dh]
  const void* K; int64_t ldk;       // [T][n_kv_heads * dh]
  const void* V; int64_t ldv;
  void* O; int64_t ldo;             // [T][n_heads * dh]
  const int32_t* cu; int S, T;
  int n_heads, group, dh;           // group = n_heads / n_kv_heads
  float scale;
  int bf16;
};
struct QkRopeArgs {
  void* Q; int64_t ldq;             // [T][n_heads * dh], in place
  void* K; int64_t ldk;             // [T][n_kv_heads * dh], in place
  const int32_t* cu; int S, T;
  int n_heads, n_kv_heads, dh;
  const float* gamma_q; const float* gamma_k;   // both null: no norm
  float eps;
  float theta;                      // <= 0: no rotation
  int bf16;
};
hipError_t launch_qk_norm_rope(const QkRopeArgs& a, hipStream_t st);

int attention_f32_max_head_dim();
int attention_bf16_head_dim();
hipError_t launch_attention(const AttnArgs& a, hipStream_t st);

}  // namespace zo
