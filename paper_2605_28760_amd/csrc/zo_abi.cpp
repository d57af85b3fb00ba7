// Host side of the C ABI declared in include/zo.h: argument validation (all of
// it before the first HIP call), workspace planning and kernel sequencing.
// The ProbePlan -> observations boundary of Sec. 2.3 (Eq. 4) is this file.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <string>

#include "../../include/zo.h"
#include "zo_host.hpp"
#include "zo_internal.hpp"

namespace zo {

// ---- launch planning of the side-down pass (host only) ------------------------------------
// K ranges per row: four ranges up to 12288 columns, ranges of about 2560 columns for wider inputs, never
// narrower than 512 columns, whole 64-column steps.  A function of the input width alone: the range a
// column falls in, and with it the order in which a row's products are summed, must not depend on the batch.
int side_ksplit(int n) {
  int s = n <= 12288 ? 4 : (n + 1280) / 2560;
  if (s > 8) s = 8;
  while (s > 1 && n / s < 512) --s;
  return s < 1 ? 1 : s;
}

// Rows per item (64, 48, 32 or 16; how rows are grouped into items does not enter any row's arithmetic).  The
// workgroups of a pass (seven or eight items each, times the K ranges) run in rounds of one workgroup per
// compute unit, and a round that is mostly empty takes as long as a full one.  A workgroup's time per K step
// has a part that grows with its items' rows (their bytes of X) and a part that does not (the V and Vb
// blocks: about two rows' worth per 16 bank columns): the size that makes rounds x time smallest, the larger
// one on a tie (it re-reads V less often).  With the host mirrors of the batch the items are counted as the
// device will build them (none for foreground sequences); without, every row counts.
int side_item_rows(const int32_t* host_cu, const int32_t* host_seq_cand, int S, int T, int n, int R) {
  const int cus = compute_units();
  const int ks = side_ksplit(n);
  const int fixed = 2 * ((R + 15) / 16);
  const int nbb = (R + 15) / 16 < kSideMaxBlocks - 1 ? (R + 15) / 16 : kSideMaxBlocks - 1;   // bank blocks of the first pass
  static const int kSizes[4] = {64, 48, 32, 16};
  int best = kSideRows;
  int64_t best_cost = -1;
  for (int rows : kSizes) {
    int64_t items = 0;
    if (host_cu && host_seq_cand) {
      for (int q = 0; q < S; ++q)
        if (host_seq_cand[q] >= 0) items += (host_cu[q + 1] - host_cu[q] + rows - 1) / rows;
    } else {
      items = (T + rows - 1) / rows;
    }
    const int w = side_waves_of(nbb, rows / 16);
    const int64_t wgs = ((items + w - 1) / w) * ks;
    const int64_t cost = ((wgs + cus - 1) / cus) * (rows + fixed);
    if (best_cost < 0 || cost < best_cost) { best = rows; best_cost = cost; }
  }
  return best;
}

}  // namespace zo

namespace {

thread_local std::string g_err;

int32_t fail(zo_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return (int32_t)st;
}

int32_t hip_fail(hipError_t e, const char* where) {
  return fail(ZO_ERR_HIP, "%s: %s", where, hipGetErrorString(e));
}

#define ZO_HIP(call, where)                              \
  do {                                                   \
    hipError_t e__ = (call);                             \
    if (e__ != hipSuccess) return hip_fail(e__, where);  \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int round16(int x) { return (x + 15) / 16 * 16; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
constexpr int64_t kMaxLd = (int64_t)1 << 22;  // keeps 256-row tile offsets inside 32 bits

// Carves 256-byte aligned regions out of the caller's workspace.
struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  }
};

int32_t check_batch(const zo_batch* b) {
  if (!b) return fail(ZO_ERR_NULL, "batch is NULL");
  if (b->n_tokens < 0 || b->n_seqs < 0 || b->n_cands < 0 || b->n_dirs < 0)
    return fail(ZO_ERR_SHAPE, "negative batch size (T=%d S=%d C=%d K=%d)", b->n_tokens, b->n_seqs, b->n_cands,
                b->n_dirs);
  if (b->n_tokens > 0 && b->n_seqs == 0) return fail(ZO_ERR_SHAPE, "n_tokens > 0 with no sequences");
  if (!b->cu_seqlens) return fail(ZO_ERR_NULL, "batch.cu_seqlens is NULL");
  if (b->n_seqs > 0 && !b->seq_cand) return fail(ZO_ERR_NULL, "batch.seq_cand is NULL");
  if (b->n_cands > 0 && (!b->cand_dir || !b->cand_sign)) return fail(ZO_ERR_NULL, "batch.cand_dir / cand_sign is NULL");
  if (b->n_dirs > 0 && !b->dir_seed) return fail(ZO_ERR_NULL, "batch.dir_seed is NULL");
  if (b->host_cu_seqlens) {
    const int32_t* cu = b->host_cu_seqlens;
    if (cu[0] != 0) return fail(ZO_ERR_INDEX, "cu_seqlens[0] = %d, expected 0", cu[0]);
    for (int s = 0; s < b->n_seqs; ++s)
      if (cu[s + 1] < cu[s]) return fail(ZO_ERR_INDEX, "cu_seqlens decreases at sequence %d", s);
    if (cu[b->n_seqs] != b->n_tokens)
      return fail(ZO_ERR_INDEX, "cu_seqlens[S] = %d but n_tokens = %d", cu[b->n_seqs], b->n_tokens);
  }
  if (b->host_seq_cand)
    for (int s = 0; s < b->n_seqs; ++s)
      if (b->host_seq_cand[s] < -1 || b->host_seq_cand[s] >= b->n_cands)
        return fail(ZO_ERR_INDEX, "seq_cand[%d] = %d outside [-1, %d)", s, b->host_seq_cand[s], b->n_cands);
  if (b->host_cand_dir)
    for (int c = 0; c < b->n_cands; ++c)
      if (b->host_cand_dir[c] < -1 || b->host_cand_dir[c] >= b->n_dirs)
        return fail(ZO_ERR_INDEX, "cand_dir[%d] = %d outside [-1, %d)", c, b->host_cand_dir[c], b->n_dirs);
  return ZO_OK;
}

zo::BatchDev to_dev(const zo_batch* b) {
  zo::BatchDev d;
  d.T = b->n_tokens; d.S = b->n_seqs; d.C = b->n_cands; d.K = b->n_dirs;
  d.cu = b->cu_seqlens; d.seq_cand = b->seq_cand; d.cand_dir = b->cand_dir; d.cand_sign = b->cand_sign;
  d.seed = b->dir_seed;
  d.seed_v = b->dir_seed_v;
  return d;
}

// ---- workspace plans --------------------------------------------------------------------
struct ProbePlan {
  int RP = 0, Rp = 0, max_items = 0, item_rows = zo::kSideRows, ksplit = 1;
  int SPD = 0, RpT = 0, n_tn = 0, slot_cap = 0, kt_cap = 0, m_img = 0;   // side K tiles of the bf16 GEMM
  size_t uimg_bytes = 0, pimg_bytes = 0, xs_bytes = 0;
  size_t seq_kind, seq_scale, tok_seq, n_items, items;
  size_t tile_hdr, tile_slots, kt_tile, Uimg, Vt, Pimg, Vbt, Xs, partial;   // bf16 path
  size_t Uf, Vf, Tside;                                                     // fp32 path
  size_t total = 0;
};

ProbePlan plan_probe(int T, int S, int K, int m, int n, int r, int R, zo_dtype dt, const int32_t* host_cu = nullptr,
                     const int32_t* host_seq_cand = nullptr) {
  ProbePlan p;
  Carver c;
  p.seq_kind = c.take((size_t)S * 4);
  p.seq_scale = c.take((size_t)S * 4);
  p.tok_seq = c.take((size_t)T * 4);
  p.n_items = c.take(16);
  // (the choice of the item size does not enter the layout below: a workspace query, which has no batch, and
  // the call agree on every offset)
  p.item_rows = dt == ZO_BF16 ? zo::side_item_rows(host_cu, host_seq_cand, S, T, n, R) : zo::kSideRows;
  p.max_items = (T + p.item_rows - 1) / p.item_rows + S;
  // (sized for the smallest items, so that a workspace sized for a large batch also serves a smaller one)
  p.items = c.take(((size_t)(T + 15) / 16 + S) * sizeof(zo::SideItem));
  if (dt == ZO_BF16) {
    p.RP = round16(r);
    p.Rp = round16(R);
    const size_t NC = (size_t)p.RP + p.Rp;
    p.ksplit = zo::side_ksplit(n);
    // Side K tiles.  A token tile's slot list holds one entry per distinct direction among the sequences
    // that intersect it (times the 32-column blocks of a direction): over all tiles at most tiles +
    // sequences, and at most min(K, 256) per tile.  A K tile holds two slots; a tile with candidates
    // also has the bank's K tiles.
    p.SPD = (r + 31) / 32;
    p.RpT = (R + zo::kTileK - 1) / zo::kTileK;
    p.n_tn = (T + zo::kTileN - 1) / zo::kTileN;
    const int64_t per_tile = K < zo::kTileN ? K : zo::kTileN;
    int64_t dirs = (int64_t)p.n_tn + S;
    if (dirs > (int64_t)p.n_tn * per_tile) dirs = (int64_t)p.n_tn * per_tile;
    p.slot_cap = (int)(dirs * p.SPD);
    p.kt_cap = (p.slot_cap + p.n_tn + 1) / 2 + p.n_tn * p.RpT;
    p.m_img = (m + zo::kTileM - 1) / zo::kTileM * zo::kTileM + zo::kTileM / 2;   // a half tile may start 128 rows down
    p.uimg_bytes = (size_t)K * p.SPD * p.m_img * 64;
    p.pimg_bytes = (size_t)p.RpT * p.m_img * 128;
    p.xs_bytes = (size_t)p.kt_cap * zo::kTileN * zo::kTileK * 2;
    p.tile_hdr = c.take((size_t)p.n_tn * sizeof(zo::TileHdr));
    p.tile_slots = c.take((size_t)p.slot_cap * 4);
    p.kt_tile = c.take((size_t)p.kt_cap * 4);
    p.Uimg = c.take(p.uimg_bytes);
    p.Vt = c.take((size_t)K * p.RP * n * 2);
    p.Pimg = c.take(p.pimg_bytes);
    p.Vbt = c.take((size_t)p.Rp * n * 2);
    p.Xs = c.take(p.xs_bytes);
    p.partial = c.take((size_t)p.ksplit * T * NC * 4);
  } else {
    p.Uf = c.take((size_t)K * m * r * 4);
    p.Vf = c.take((size_t)K * n * r * 4);
    p.Tside = c.take((size_t)T * (r + R) * 4);
  }
  p.total = c.off;
  return p;
}

struct ScorePlan {
  int n_vt = 0;
  size_t part_max, part_sum, tgt_logit, tok_nll, seq_cnt, rows, pos, n_rows, total = 0;
};

ScorePlan plan_score(int T, int S, int vocab, zo_dtype dt) {
  ScorePlan p;
  Carver c;
  p.n_vt = dt == ZO_BF16 ? zo::head_vocab_tiles_bf16(vocab) : zo::head_vocab_tiles_f32(vocab);
  p.part_max = c.take((size_t)p.n_vt * T * 4);
  p.part_sum = c.take((size_t)p.n_vt * T * 4);
  p.tgt_logit = c.take((size_t)T * 4);
  p.tok_nll = c.take((size_t)T * 4);
  p.seq_cnt = c.take((size_t)S * 4);
  p.rows = c.take((size_t)T * 4);     // list of scored tokens
  p.pos = c.take((size_t)T * 4);      // position of a token in that list
  p.n_rows = c.take(16);
  p.total = c.off;
  return p;
}

bool ld_too_small(int64_t ld, int cols) { return ld < cols || ld > kMaxLd; }

int32_t check_matrix(const char* name, const void* p, int64_t ld, int cols, zo_dtype dt) {
  if (ld < cols || ld > kMaxLd) return fail(ZO_ERR_SHAPE, "%s: leading dimension %lld invalid for %d columns", name, (long long)ld, cols);
  if (dt == ZO_BF16) {
    if (!aligned16(p)) return fail(ZO_ERR_SHAPE, "%s: pointer not 16-byte aligned", name);
    if (ld % 8 != 0) return fail(ZO_ERR_SHAPE, "%s: leading dimension %lld does not keep rows 16-byte aligned", name, (long long)ld);
  } else if (((uintptr_t)p & 3u) != 0) {
    return fail(ZO_ERR_SHAPE, "%s: pointer not 4-byte aligned", name);
  }
  return ZO_OK;
}

}  // namespace

extern "C" {

int32_t zo_version(void) { return 1000; }

size_t zo_last_error(char* buf, size_t cap) {
  if (buf && cap > 0) {
    const size_t n = g_err.size() < cap - 1 ? g_err.size() : cap - 1;
    memcpy(buf, g_err.data(), n);
    buf[n] = 0;
  }
  return g_err.size();
}

int32_t zo_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t first_block, int64_t n_blocks,
                        uint32_t* out_words, void* stream) {
  if (n_blocks < 0) return fail(ZO_ERR_SHAPE, "n_blocks = %lld", (long long)n_blocks);
  if (n_blocks == 0) return ZO_OK;
  if (!out_words) return fail(ZO_ERR_NULL, "out_words is NULL");
  if (!aligned16(out_words)) return fail(ZO_ERR_SHAPE, "out_words not 16-byte aligned");
  ZO_HIP(zo::launch_philox_words(seed, tensor_id, first_block, n_blocks, out_words, (hipStream_t)stream), "zo_philox_words");
  return ZO_OK;
}

int32_t zo_factor_fill(uint64_t seed, uint32_t tensor_id, int64_t rows, int32_t r, zo_dtype dtype, void* out,
                       void* stream) {
  if (rows < 0 || r < 1) return fail(ZO_ERR_SHAPE, "rows = %lld, r = %d", (long long)rows, r);
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  if (rows == 0) return ZO_OK;
  if (!out) return fail(ZO_ERR_NULL, "out is NULL");
  ZO_HIP(zo::launch_factor_fill(seed, tensor_id, rows, r, dtype == ZO_BF16, out, (hipStream_t)stream), "zo_factor_fill");
  return ZO_OK;
}

int32_t zo_batch_index(const zo_batch* batch, int32_t* tok_seq, int32_t* tok_cand, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (batch->n_tokens == 0) return ZO_OK;
  ZO_HIP(zo::launch_tok_index(to_dev(batch), tok_seq, tok_cand, (hipStream_t)stream), "zo_batch_index");
  return ZO_OK;
}

size_t zo_probe_linear_workspace_bytes(int32_t n_tokens, int32_t n_seqs, int32_t n_dirs, int32_t m, int32_t n,
                                       int32_t r, int32_t R_used, zo_dtype in_dtype) {
  if (n_tokens < 0 || n_seqs < 0 || n_dirs < 0 || m < 0 || n < 0 || r < 0 || R_used < 0) return 0;
  return plan_probe(n_tokens, n_seqs, n_dirs, m, n, r, R_used, in_dtype).total;
}

int32_t zo_probe_linear(const zo_batch* batch, const void* X, int64_t ldx, const void* W, int64_t ldw,
                        const float* bias, int32_t m, int32_t n, zo_dtype in_dtype, int32_t r, float eps,
                        uint32_t tensor_id, const zo_bank* bank, int32_t act, void* Y, int64_t ldy,
                        zo_dtype out_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (m < 0 || n < 0) return fail(ZO_ERR_SHAPE, "m = %d, n = %d", m, n);
  if (r < 1 || r > zo::kMaxRank) return fail(ZO_ERR_SHAPE, "rank r = %d outside [1, %d]", r, zo::kMaxRank);
  if (in_dtype != ZO_F32 && in_dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "in_dtype %d", (int)in_dtype);
  if (!(out_dtype == in_dtype || (in_dtype == ZO_BF16 && out_dtype == ZO_F32)))
    return fail(ZO_ERR_UNSUPPORTED, "in_dtype %d with out_dtype %d", (int)in_dtype, (int)out_dtype);
  if (act < 0 || act > 2) return fail(ZO_ERR_UNSUPPORTED, "activation %d", act);
  if (act == 2 && m % 2 != 0) return fail(ZO_ERR_SHAPE, "the gated activation pairs output features: m = %d is odd", m);
  const int m_out = act == 2 ? m / 2 : m;   // columns of Y
  const int T = batch->n_tokens;
  int R = 0;
  if (bank) {
    if (bank->R_cap < 0 || bank->R_used < 0 || bank->R_used > bank->R_cap)
      return fail(ZO_ERR_SHAPE, "bank R_used = %d, R_cap = %d", bank->R_used, bank->R_cap);
    R = bank->R_used;
    if (R > 0 && (!bank->P || !bank->Vb)) return fail(ZO_ERR_NULL, "bank.P / bank.Vb is NULL");
  }
  if (T == 0 || m == 0) return ZO_OK;
  if (!X || !W || !Y) return fail(ZO_ERR_NULL, "X, W or Y is NULL");
  if (int32_t st = check_matrix("X", X, ldx, n, in_dtype)) return st;
  if (int32_t st = check_matrix("W", W, ldw, n, in_dtype)) return st;
  if (int32_t st = check_matrix("Y", Y, ldy, m_out, out_dtype)) return st;
  if (in_dtype == ZO_BF16 && (n % zo::kTileK != 0 || n == 0))
    return fail(ZO_ERR_UNSUPPORTED, "bf16 path needs n %% %d == 0 (n = %d)", zo::kTileK, n);
  if (out_dtype == ZO_BF16 && m_out % 8 != 0)
    return fail(ZO_ERR_UNSUPPORTED, "bf16 output needs a multiple of 8 output columns (m = %d, activation %d)", m, act);
  const ProbePlan plan = plan_probe(T, batch->n_seqs, batch->n_dirs, m, n, r, R, in_dtype, batch->host_cu_seqlens,
                                    batch->host_seq_cand);
  if (!workspace) return fail(ZO_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", plan.total);
  if (((uintptr_t)workspace & 255u) != 0) return fail(ZO_ERR_WORKSPACE, "workspace not 256-byte aligned");
  if (workspace_bytes < plan.total)
    return fail(ZO_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.total);

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const zo::BatchDev bd = to_dev(batch);
  zo::SeqTables tabs;
  tabs.seq_kind = (int32_t*)(ws + plan.seq_kind);
  tabs.seq_scale = (float*)(ws + plan.seq_scale);
  tabs.tok_seq = (int32_t*)(ws + plan.tok_seq);
  tabs.items = (zo::SideItem*)(ws + plan.items);
  tabs.n_items = (int32_t*)(ws + plan.n_items);
  tabs.max_items = plan.max_items;
  tabs.item_rows = plan.item_rows;
  tabs.tile_hdr = nullptr; tabs.tile_slots = nullptr; tabs.kt_tile = nullptr;
  tabs.n_tn = plan.n_tn; tabs.slot_cap = plan.slot_cap; tabs.kt_cap = plan.kt_cap; tabs.SPD = plan.SPD; tabs.RpT = plan.RpT;
  // a batch without candidates (or probes and bank both absent) is a plain GEMM
  const bool has_side = batch->n_cands > 0;
  if (has_side && in_dtype != ZO_BF16) ZO_HIP(zo::launch_seq_tables(bd, eps, tabs, st), "batch tables");

  if (in_dtype == ZO_BF16) {
    uint16_t* Uimg = (uint16_t*)(ws + plan.Uimg);
    uint16_t* Vt = (uint16_t*)(ws + plan.Vt);
    uint16_t* Pimg = (uint16_t*)(ws + plan.Pimg);
    uint16_t* Vbt = (uint16_t*)(ws + plan.Vbt);
    uint16_t* Xs = (uint16_t*)(ws + plan.Xs);
    if (has_side) {
      // the GEMM addresses each image through one buffer window with 31-bit offsets
      const size_t window = (size_t)0x7FFFFFFF;
      if (plan.uimg_bytes > window || plan.pimg_bytes > window || plan.xs_bytes > window)
        return fail(ZO_ERR_UNSUPPORTED, "side-state images of %zu / %zu / %zu bytes exceed the 2 GiB addressing window "
                    "(directions x rank x output features, bank rank x output features, tokens x side columns)",
                    plan.uimg_bytes, plan.pimg_bytes, plan.xs_bytes);
      tabs.tile_hdr = (zo::TileHdr*)(ws + plan.tile_hdr);
      tabs.tile_slots = (int32_t*)(ws + plan.tile_slots);
      tabs.kt_tile = (int32_t*)(ws + plan.kt_tile);
      ZO_HIP(zo::launch_probe_prep_bf16(bd, eps, tabs, tensor_id, m, n, r, plan.RP, plan.Rp, R > 0 ? bank->P : nullptr,
                                        R > 0 ? bank->Vb : nullptr, R > 0 ? bank->R_cap : 0, R, plan.m_img, Uimg, Vt, Pimg,
                                        Vbt, st),
             "probe preparation");
      zo::SideDownArgs sd;
      sd.X = (const uint16_t*)X; sd.ldx = ldx; sd.Vt = Vt; sd.Vbt = Vbt;
      sd.n = n; sd.RP = plan.RP; sd.Rp = plan.Rp; sd.T = T;
      sd.items = tabs.items; sd.n_items = tabs.n_items; sd.max_items = plan.max_items; sd.item_rows = plan.item_rows;
      sd.ksplit = plan.ksplit; sd.partial = (float*)(ws + plan.partial);
      sd.tok_seq = tabs.tok_seq; sd.seq_kind = tabs.seq_kind; sd.seq_scale = tabs.seq_scale;
      sd.tile_hdr = tabs.tile_hdr; sd.tile_slots = tabs.tile_slots; sd.kt_tile = tabs.kt_tile;
      sd.kt_cap = plan.kt_cap; sd.SPD = plan.SPD; sd.Xs = Xs;
      ZO_HIP(zo::launch_side_down_bf16(sd, st), "side-down");
    }
    zo::ProbeGemmArgs g;
    g.X = (const uint16_t*)X; g.ldx = ldx; g.W = (const uint16_t*)W; g.ldw = ldw; g.bias = bias;
    g.T = T; g.m = m; g.n = n; g.act = act; g.Y = Y; g.ldy = ldy; g.out_bf16 = out_dtype == ZO_BF16;
    g.has_side = has_side; g.tile_hdr = tabs.tile_hdr; g.tile_slots = tabs.tile_slots;
    g.Uimg = Uimg; g.Pimg = Pimg; g.Xs = Xs; g.m_img = plan.m_img;
    g.uimg_bytes = (int64_t)plan.uimg_bytes; g.pimg_bytes = (int64_t)plan.pimg_bytes; g.xs_bytes = (int64_t)plan.xs_bytes;
    ZO_HIP(zo::launch_probe_gemm_bf16(g, st), "probe GEMM");
  } else {
    zo::ProbeF32Args a;
    a.X = (const float*)X; a.ldx = ldx; a.W = (const float*)W; a.ldw = ldw; a.bias = bias;
    a.T = T; a.m = m; a.n = n; a.r = r; a.R = R; a.R_cap = bank ? bank->R_cap : 0; a.act = act;
    a.Y = (float*)Y; a.ldy = ldy; a.has_side = has_side;
    a.tok_seq = tabs.tok_seq; a.seq_kind = tabs.seq_kind; a.seq_scale = tabs.seq_scale;
    a.Uf = (float*)(ws + plan.Uf); a.Vf = (float*)(ws + plan.Vf);
    a.P = bank ? bank->P : nullptr; a.Vb = bank ? bank->Vb : nullptr;
    a.Tside = (float*)(ws + plan.Tside);
    if (has_side) ZO_HIP(zo::launch_factors_f32(bd, tensor_id, m, n, r, (float*)(ws + plan.Uf), (float*)(ws + plan.Vf), st), "fp32 factors");
    ZO_HIP(zo::launch_probe_f32(a, st), "fp32 probe linear");
  }
  return ZO_OK;
}

size_t zo_score_workspace_bytes(int32_t n_tokens, int32_t n_seqs, int32_t vocab, int32_t d, zo_dtype dtype) {
  (void)d;
  if (n_tokens < 0 || n_seqs < 0 || vocab < 0) return 0;
  return plan_score(n_tokens, n_seqs, vocab, dtype).total;
}

}  // extern "C"

// Everything zo_score checks before it looks at its workspace (no HIP call).
int32_t zo::score_validate(const zo_batch* batch, const void* H, int64_t ldh, const void* W_head, int64_t ldw,
                           int32_t vocab, int32_t d, zo_dtype dtype, const int32_t* targets, const float* seq_nll,
                           const float* cand_sum, const int32_t* cand_cnt) {
  if (int32_t st = check_batch(batch)) return st;
  if (vocab < 1 || d < 1) return fail(ZO_ERR_SHAPE, "vocab = %d, d = %d", vocab, d);
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  const int T = batch->n_tokens, S = batch->n_seqs, C = batch->n_cands;
  if (S > 0 && !seq_nll) return fail(ZO_ERR_NULL, "seq_nll is NULL");
  if (C > 0 && (!cand_sum || !cand_cnt)) return fail(ZO_ERR_NULL, "cand_sum / cand_cnt is NULL");
  if (T > 0) {
    if (!H || !W_head || !targets) return fail(ZO_ERR_NULL, "H, W_head or targets is NULL");
    if (int32_t st = check_matrix("H", H, ldh, d, dtype)) return st;
    if (int32_t st = check_matrix("W_head", W_head, ldw, d, dtype)) return st;
    if (dtype == ZO_BF16 && d % zo::kTileK != 0)
      return fail(ZO_ERR_UNSUPPORTED, "bf16 path needs d %% %d == 0 (d = %d)", zo::kTileK, d);
  }
  return ZO_OK;
}

int32_t zo::fail_status(int32_t status, const char* message) { return fail((zo_status)status, "%s", message); }

extern "C" {

int32_t zo_score(const zo_batch* batch, const void* H, int64_t ldh, const void* W_head, int64_t ldw,
                 int32_t vocab, int32_t d, zo_dtype dtype, const int32_t* targets, float* tok_nll,
                 float* seq_nll, float* cand_sum, int32_t* cand_cnt, void* workspace, size_t workspace_bytes,
                 void* stream) {
  if (int32_t st = zo::score_validate(batch, H, ldh, W_head, ldw, vocab, d, dtype, targets, seq_nll, cand_sum, cand_cnt))
    return st;
  const int T = batch->n_tokens, S = batch->n_seqs, C = batch->n_cands;
  const ScorePlan plan = plan_score(T, S, vocab, dtype);
  if (plan.total > 0) {
    if (!workspace) return fail(ZO_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", plan.total);
    if (((uintptr_t)workspace & 255u) != 0) return fail(ZO_ERR_WORKSPACE, "workspace not 256-byte aligned");
    if (workspace_bytes < plan.total)
      return fail(ZO_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.total);
  }
  if (S == 0 && C == 0) return ZO_OK;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* part_max = (float*)(ws + plan.part_max);
  float* part_sum = (float*)(ws + plan.part_sum);
  float* tgt = (float*)(ws + plan.tgt_logit);
  const int32_t* pos = nullptr;
  if (T > 0) {
    if (dtype == ZO_BF16) {
      zo::HeadScoreArgs a;
      a.H = (const uint16_t*)H; a.ldh = ldh; a.Wh = (const uint16_t*)W_head; a.ldw = ldw;
      a.T = T; a.vocab = vocab; a.d = d; a.targets = targets;
      a.part_max = part_max; a.part_sum = part_sum; a.tgt_logit = tgt;
      a.rows = nullptr; a.n_rows = nullptr;
      // Only tokens with a target need logits: the head multiplies the rows of a device-built list of
      // them.  The list addresses H through one 2 GiB buffer window; a larger H is multiplied whole.
      if (((int64_t)(T - 1) * ldh + d) * 2 < ((int64_t)1 << 31)) {
        int32_t* rows = (int32_t*)(ws + plan.rows);
        ZO_HIP(zo::launch_active_rows(targets, T, rows, (int32_t*)(ws + plan.pos), (int32_t*)(ws + plan.n_rows), st),
               "scored-token list");
        a.rows = rows; a.n_rows = (const int32_t*)(ws + plan.n_rows);
        pos = (const int32_t*)(ws + plan.pos);
      }
      ZO_HIP(zo::launch_head_score_bf16(a, st), "head scoring");
    } else {
      zo::HeadScoreF32Args a;
      a.H = (const float*)H; a.ldh = ldh; a.Wh = (const float*)W_head; a.ldw = ldw;
      a.T = T; a.vocab = vocab; a.d = d; a.targets = targets;
      a.part_max = part_max; a.part_sum = part_sum; a.tgt_logit = tgt;
      ZO_HIP(zo::launch_head_score_f32(a, st), "fp32 head scoring");
    }
  }
  zo::ScoreCombineArgs c;
  c.T = T; c.S = S; c.C = C; c.n_vt = plan.n_vt;
  c.part_max = part_max; c.part_sum = part_sum; c.tgt_logit = tgt; c.targets = targets; c.pos = pos;
  c.cu = batch->cu_seqlens; c.seq_cand = batch->seq_cand;
  c.tok_nll = tok_nll ? tok_nll : (float*)(ws + plan.tok_nll);
  c.seq_nll = seq_nll; c.seq_cnt = (int32_t*)(ws + plan.seq_cnt);
  c.cand_sum = cand_sum; c.cand_cnt = cand_cnt;
  ZO_HIP(zo::launch_score_combine(c, st), "score combine");
  return ZO_OK;
}

int32_t zo_estimate(const zo_batch* batch, const float* cand_sum, const int32_t* cand_cnt, float eps,
                    int32_t reduction, float* cand_loss, float* proj_grad, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (reduction != 0 && reduction != 1) return fail(ZO_ERR_UNSUPPORTED, "reduction %d", reduction);
  if (!(eps > 0.0f)) return fail(ZO_ERR_SHAPE, "eps = %g must be positive", (double)eps);
  if (batch->n_cands > 0 && (!cand_sum || !cand_cnt || !cand_loss)) return fail(ZO_ERR_NULL, "cand_sum, cand_cnt or cand_loss is NULL");
  if (batch->n_dirs > 0 && !proj_grad) return fail(ZO_ERR_NULL, "proj_grad is NULL");
  ZO_HIP(zo::launch_estimate(to_dev(batch), cand_sum, cand_cnt, eps, reduction, cand_loss, proj_grad, (hipStream_t)stream), "zo_estimate");
  return ZO_OK;
}

int32_t zo_estimate_es(const zo_batch* batch, const float* cand_sum, const int32_t* cand_cnt, float eps,
                       int32_t reduction, float* cand_loss, float* proj_grad, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (reduction != 0 && reduction != 1) return fail(ZO_ERR_UNSUPPORTED, "reduction %d", reduction);
  if (!(eps > 0.0f)) return fail(ZO_ERR_SHAPE, "eps = %g must be positive", (double)eps);
  if (batch->n_cands > 0 && (!cand_sum || !cand_cnt || !cand_loss)) return fail(ZO_ERR_NULL, "cand_sum, cand_cnt or cand_loss is NULL");
  if (batch->n_dirs > 0 && !proj_grad) return fail(ZO_ERR_NULL, "proj_grad is NULL");
  ZO_HIP(zo::launch_estimate_es(to_dev(batch), cand_sum, cand_cnt, eps, reduction, cand_loss, proj_grad, (hipStream_t)stream), "zo_estimate_es");
  return ZO_OK;
}

namespace {
int32_t check_bank_update(const zo_bank* bank, int32_t m, int32_t n, int32_t r, int32_t n_dirs, zo_dtype factor_dtype) {
  if (!bank) return fail(ZO_ERR_NULL, "bank is NULL");
  if (m < 0 || n < 0 || n_dirs < 0) return fail(ZO_ERR_SHAPE, "m = %d, n = %d, n_dirs = %d", m, n, n_dirs);
  if (r < 1 || r > zo::kMaxRank) return fail(ZO_ERR_SHAPE, "rank r = %d outside [1, %d]", r, zo::kMaxRank);
  if (bank->R_cap < 0 || bank->R_used < 0 || bank->R_used > bank->R_cap)
    return fail(ZO_ERR_SHAPE, "bank R_used = %d, R_cap = %d", bank->R_used, bank->R_cap);
  if (factor_dtype != ZO_F32 && factor_dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "factor_dtype %d", (int)factor_dtype);
  return ZO_OK;
}

// The column blocks [col0[k], col0[k] + r) of the directions: inside the bank, pairwise disjoint, and
// when accumulating, inside the columns in use.  *new_used = R_used after an append.
int32_t check_col_blocks(const zo_bank* bank, int32_t r, int32_t n_dirs, const int32_t* host_col0, int32_t append,
                         int* new_used) {
  *new_used = bank->R_used;
  for (int k = 0; k < n_dirs; ++k) {
    const int c0 = host_col0[k];
    if (c0 < 0) return fail(ZO_ERR_SHAPE, "col0[%d] = %d", k, c0);
    if (c0 + r > bank->R_cap) return fail(ZO_ERR_BANK_FULL, "direction %d: columns [%d, %d) exceed R_cap = %d", k, c0, c0 + r, bank->R_cap);
    if (!append && c0 + r > bank->R_used)
      return fail(ZO_ERR_SHAPE, "direction %d accumulates into columns [%d, %d) beyond R_used = %d", k, c0, c0 + r, bank->R_used);
    for (int j = 0; j < k; ++j)
      if (c0 < host_col0[j] + r && host_col0[j] < c0 + r)
        return fail(ZO_ERR_SHAPE, "column blocks of directions %d and %d overlap", j, k);
    if (c0 + r > *new_used) *new_used = c0 + r;
  }
  return ZO_OK;
}
}  // namespace

int32_t zo_bank_update(zo_bank* bank, int32_t m, int32_t n, int32_t r, int32_t n_dirs, const uint64_t* dir_seed,
                       const uint64_t* dir_seed_v, uint32_t tensor_id, const float* proj_grad, float lr,
                       const float* dir_weight, const int32_t* host_col0, int32_t append, zo_dtype factor_dtype,
                       void* stream) {
  if (int32_t st = check_bank_update(bank, m, n, r, n_dirs, factor_dtype)) return st;
  if (append != 0 && append != 1) return fail(ZO_ERR_UNSUPPORTED, "append = %d", append);
  if (n_dirs == 0) return ZO_OK;
  if (!dir_seed || !proj_grad || !host_col0) return fail(ZO_ERR_NULL, "dir_seed, proj_grad or host_col0 is NULL");
  if (!bank->P || (append && !bank->Vb)) return fail(ZO_ERR_NULL, "bank.P / bank.Vb is NULL");
  int new_used = 0;
  if (int32_t st = check_col_blocks(bank, r, n_dirs, host_col0, append, &new_used)) return st;
  zo::BankUpdateArgs a;
  a.P = bank->P; a.Vb = bank->Vb; a.R_cap = bank->R_cap; a.m = m; a.n = n; a.r = r;
  a.seed = dir_seed; a.seed_v = dir_seed_v; a.tensor_id = tensor_id; a.proj_grad = proj_grad; a.lr = lr;
  a.dir_weight = dir_weight; a.sched = nullptr; a.n_dirs = n_dirs;
  a.default_weight = 1.0f / (float)n_dirs; a.append = append; a.bf16 = factor_dtype == ZO_BF16;
  ZO_HIP(zo::launch_bank_update(a, n_dirs, host_col0, (hipStream_t)stream), "zo_bank_update");
  if (append) bank->R_used = new_used;
  return ZO_OK;
}

int32_t zo_bank_update_multi(zo_layer_bank* layers, int32_t n_layers, int32_t r, int32_t n_dirs,
                             const uint64_t* dir_seed, const uint64_t* dir_seed_v, const float* proj_grad, float lr,
                             const float* dir_weight, const int32_t* host_col0, int32_t append,
                             zo_dtype factor_dtype, void* stream) {
  if (n_layers < 0) return fail(ZO_ERR_SHAPE, "n_layers = %d", n_layers);
  if (n_layers > 0 && !layers) return fail(ZO_ERR_NULL, "layers is NULL");
  if (append != 0 && append != 1) return fail(ZO_ERR_UNSUPPORTED, "append = %d", append);
  // everything is validated before the first launch
  for (int i = 0; i < n_layers; ++i)
    if (int32_t st = check_bank_update(&layers[i].bank, layers[i].m, layers[i].n, r, n_dirs, factor_dtype)) return st;
  if (n_layers == 0 || n_dirs == 0) return ZO_OK;
  if (!dir_seed || !proj_grad || !host_col0) return fail(ZO_ERR_NULL, "dir_seed, proj_grad or host_col0 is NULL");
  for (int i = 0; i < n_layers; ++i) {
    const zo_bank* b = &layers[i].bank;
    int new_used = 0;
    if (!b->P || (append && !b->Vb)) return fail(ZO_ERR_NULL, "layer %d: bank.P / bank.Vb is NULL", i);
    if (int32_t st = check_col_blocks(b, r, n_dirs, host_col0, append, &new_used)) return st;
  }
  zo::BankUpdateArgs a;   // what the layers share; the per-layer fields are filled in on the device
  a.P = nullptr; a.Vb = nullptr; a.R_cap = 0; a.m = 0; a.n = 0; a.tensor_id = 0; a.r = r;
  a.seed = dir_seed; a.seed_v = dir_seed_v; a.proj_grad = proj_grad; a.lr = lr;
  a.dir_weight = dir_weight; a.sched = nullptr; a.n_dirs = n_dirs;
  a.default_weight = 1.0f / (float)n_dirs; a.append = append; a.bf16 = factor_dtype == ZO_BF16;
  constexpr int kChunk = 192;
  zo::BankLayer chunk[kChunk];
  for (int l0 = 0; l0 < n_layers; l0 += kChunk) {
    const int nl = n_layers - l0 < kChunk ? n_layers - l0 : kChunk;
    for (int i = 0; i < nl; ++i) {
      const zo_layer_bank& l = layers[l0 + i];
      chunk[i] = zo::BankLayer{l.bank.P, l.bank.Vb, l.bank.R_cap, l.m, l.n, l.tensor_id};
    }
    ZO_HIP(zo::launch_bank_update_multi(a, chunk, nl, n_dirs, host_col0, (hipStream_t)stream), "zo_bank_update_multi");
  }
  if (append)
    for (int i = 0; i < n_layers; ++i) {
      int new_used = 0;
      check_col_blocks(&layers[i].bank, r, n_dirs, host_col0, append, &new_used);
      layers[i].bank.R_used = new_used;
    }
  return ZO_OK;
}

int32_t zo_schedule_step(zo_sched* sched, int32_t nu, int32_t n_blocks, int32_t n_dirs, uint64_t base_u,
                         uint64_t base_v, uint64_t* dir_seed, uint64_t* dir_seed_v, void* stream) {
  static_assert(sizeof(zo_sched) == sizeof(zo::SchedDev), "schedule state layouts differ");
  if (!sched) return fail(ZO_ERR_NULL, "sched is NULL");
  if (nu < 1 || n_blocks < 1 || n_dirs < 0) return fail(ZO_ERR_SHAPE, "nu = %d, n_blocks = %d, n_dirs = %d", nu, n_blocks, n_dirs);
  if (n_dirs > 0 && (!dir_seed || !dir_seed_v)) return fail(ZO_ERR_NULL, "dir_seed or dir_seed_v is NULL");
  ZO_HIP(zo::launch_schedule_step((zo::SchedDev*)sched, nu, n_blocks, n_dirs, base_u, base_v, dir_seed, dir_seed_v,
                                  (hipStream_t)stream), "zo_schedule_step");
  return ZO_OK;
}

int32_t zo_bank_update_scheduled(zo_bank* bank, int32_t m, int32_t n, int32_t r, int32_t n_dirs,
                                 const uint64_t* dir_seed, const uint64_t* dir_seed_v, uint32_t tensor_id,
                                 const float* proj_grad, float lr, const float* dir_weight, const zo_sched* sched,
                                 int32_t n_blocks, zo_dtype factor_dtype, void* stream) {
  if (int32_t st = check_bank_update(bank, m, n, r, n_dirs, factor_dtype)) return st;
  if (n_blocks < 1) return fail(ZO_ERR_SHAPE, "n_blocks = %d", n_blocks);
  if (n_dirs == 0) return ZO_OK;
  if (!dir_seed || !proj_grad || !sched) return fail(ZO_ERR_NULL, "dir_seed, proj_grad or sched is NULL");
  if (!bank->P || !bank->Vb) return fail(ZO_ERR_NULL, "bank.P / bank.Vb is NULL");
  const int64_t cols = (int64_t)n_blocks * n_dirs * r;
  if (cols > bank->R_cap)
    return fail(ZO_ERR_BANK_FULL, "%d blocks x %d directions x rank %d = %lld columns exceed R_cap = %d", n_blocks, n_dirs, r, (long long)cols, bank->R_cap);
  if (cols > bank->R_used)
    return fail(ZO_ERR_SHAPE, "scheduled updates need R_used >= %lld (all blocks in use from the start), R_used = %d", (long long)cols, bank->R_used);
  zo::BankUpdateArgs a;
  a.P = bank->P; a.Vb = bank->Vb; a.R_cap = bank->R_cap; a.m = m; a.n = n; a.r = r;
  a.seed = dir_seed; a.seed_v = dir_seed_v; a.tensor_id = tensor_id; a.proj_grad = proj_grad; a.lr = lr;
  a.dir_weight = dir_weight; a.sched = (const zo::SchedDev*)sched; a.n_dirs = n_dirs;
  a.default_weight = 1.0f / (float)n_dirs; a.append = 0; a.bf16 = factor_dtype == ZO_BF16;
  ZO_HIP(zo::launch_bank_update(a, n_dirs, nullptr, (hipStream_t)stream), "zo_bank_update_scheduled");
  return ZO_OK;
}

int32_t zo_fold_bank(zo_bank* bank, void* W, int64_t ldw, int32_t m, int32_t n, zo_dtype dtype, void* stream) {
  if (!bank) return fail(ZO_ERR_NULL, "bank is NULL");
  if (m < 0 || n < 0) return fail(ZO_ERR_SHAPE, "m = %d, n = %d", m, n);
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  if (bank->R_cap < 0 || bank->R_used < 0 || bank->R_used > bank->R_cap)
    return fail(ZO_ERR_SHAPE, "bank R_used = %d, R_cap = %d", bank->R_used, bank->R_cap);
  if (m == 0 || n == 0 || bank->R_used == 0) return ZO_OK;
  if (!W || !bank->P || !bank->Vb) return fail(ZO_ERR_NULL, "W, bank.P or bank.Vb is NULL");
  if (ld_too_small(ldw, n)) return fail(ZO_ERR_SHAPE, "W: leading dimension %lld invalid for %d columns", (long long)ldw, n);
  if (((uintptr_t)W & (dtype == ZO_BF16 ? 1u : 3u)) != 0) return fail(ZO_ERR_SHAPE, "W: pointer misaligned");
  zo::FoldArgs a;
  a.P = bank->P; a.Vb = bank->Vb; a.R_cap = bank->R_cap; a.R = bank->R_used;
  a.W = W; a.ldw = ldw; a.m = m; a.n = n; a.bf16 = dtype == ZO_BF16;
  ZO_HIP(zo::launch_fold_bank(a, (hipStream_t)stream), "zo_fold_bank");
  return ZO_OK;
}

int32_t zo_add_norm(const void* X, int64_t ldx, const void* R, int64_t ldr, const float* gamma, const float* beta,
                    int32_t kind, float norm_eps, int32_t n_tokens, int32_t d, zo_dtype dtype, void* Hsum,
                    int64_t ldh, void* Y, int64_t ldy, void* stream) {
  if (n_tokens < 0 || d < 0) return fail(ZO_ERR_SHAPE, "n_tokens = %d, d = %d", n_tokens, d);
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  if (kind != ZO_LAYER_NORM && kind != ZO_RMS_NORM) return fail(ZO_ERR_UNSUPPORTED, "normalisation kind %d", kind);
  if (!(norm_eps >= 0.0f)) return fail(ZO_ERR_SHAPE, "norm_eps = %g", (double)norm_eps);
  if (!Hsum && !Y) return fail(ZO_ERR_NULL, "Hsum and Y are both NULL: nothing to compute");
  if (Hsum && !R) return fail(ZO_ERR_NULL, "Hsum given without a residual R");
  if (n_tokens == 0 || d == 0) return ZO_OK;
  if (!X) return fail(ZO_ERR_NULL, "X is NULL");
  if (Y && !gamma) return fail(ZO_ERR_NULL, "gamma is NULL");
  const uintptr_t elem_mask = dtype == ZO_BF16 ? 1u : 3u;
  struct { const char* name; const void* p; int64_t ld; } mats[] = {
      {"X", X, ldx}, {"R", R, ldr}, {"Hsum", Hsum, ldh}, {"Y", Y, ldy}};
  for (const auto& mt : mats) {
    if (!mt.p) continue;
    if (ld_too_small(mt.ld, d))
      return fail(ZO_ERR_SHAPE, "%s: leading dimension %lld invalid for %d columns", mt.name, (long long)mt.ld, d);
    if (((uintptr_t)mt.p & elem_mask) != 0) return fail(ZO_ERR_SHAPE, "%s: pointer misaligned", mt.name);
  }
  zo::NormArgs a;
  a.X = X; a.ldx = ldx; a.R = R; a.ldr = ldr; a.gamma = gamma; a.beta = beta; a.kind = kind; a.eps = norm_eps;
  a.T = n_tokens; a.d = d; a.bf16 = dtype == ZO_BF16; a.Hsum = Hsum; a.ldh = ldh; a.Y = Y; a.ldy = ldy;
  ZO_HIP(zo::launch_add_norm(a, (hipStream_t)stream), "zo_add_norm");
  return ZO_OK;
}

int32_t zo_attention(const zo_batch* batch, const void* Q, int64_t ldq, const void* K, int64_t ldk, const void* V,
                     int64_t ldv, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, float scale,
                     zo_dtype dtype, void* O, int64_t ldo, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  if (n_heads < 1 || n_kv_heads < 1 || head_dim < 1 || n_heads > 65535)
    return fail(ZO_ERR_SHAPE, "n_heads = %d, n_kv_heads = %d, head_dim = %d", n_heads, n_kv_heads, head_dim);
  if (n_heads % n_kv_heads != 0)
    return fail(ZO_ERR_SHAPE, "n_heads = %d is not a multiple of n_kv_heads = %d", n_heads, n_kv_heads);
  if (dtype == ZO_BF16 && head_dim != zo::attention_bf16_head_dim())
    return fail(ZO_ERR_UNSUPPORTED, "the bf16 kernel covers head_dim %d only (head_dim = %d)",
                zo::attention_bf16_head_dim(), head_dim);
  if (dtype == ZO_F32 && head_dim > zo::attention_f32_max_head_dim())
    return fail(ZO_ERR_UNSUPPORTED, "the fp32 kernel covers head_dim <= %d (head_dim = %d)",
                zo::attention_f32_max_head_dim(), head_dim);
  if ((int64_t)n_heads * head_dim > kMaxLd) return fail(ZO_ERR_SHAPE, "n_heads * head_dim too large");
  if (batch->n_tokens == 0) return ZO_OK;
  if (!Q || !K || !V || !O) return fail(ZO_ERR_NULL, "Q, K, V or O is NULL");
  if (int32_t st = check_matrix("Q", Q, ldq, n_heads * head_dim, dtype)) return st;
  if (int32_t st = check_matrix("K", K, ldk, n_kv_heads * head_dim, dtype)) return st;
  if (int32_t st = check_matrix("V", V, ldv, n_kv_heads * head_dim, dtype)) return st;
  if (int32_t st = check_matrix("O", O, ldo, n_heads * head_dim, dtype)) return st;
  zo::AttnArgs a;
  a.Q = Q; a.ldq = ldq; a.K = K; a.ldk = ldk; a.V = V; a.ldv = ldv; a.O = O; a.ldo = ldo;
  a.cu = batch->cu_seqlens; a.S = batch->n_seqs; a.T = batch->n_tokens;
  a.n_heads = n_heads; a.group = n_heads / n_kv_heads; a.dh = head_dim; a.scale = scale; a.bf16 = dtype == ZO_BF16;
  ZO_HIP(zo::launch_attention(a, (hipStream_t)stream), "zo_attention");
  return ZO_OK;
}

int32_t zo_qk_norm_rope(const zo_batch* batch, void* Q, int64_t ldq, void* K, int64_t ldk, int32_t n_heads,
                        int32_t n_kv_heads, int32_t head_dim, const float* gamma_q, const float* gamma_k,
                        float norm_eps, float rope_theta, zo_dtype dtype, void* stream) {
  if (int32_t st = check_batch(batch)) return st;
  if (dtype != ZO_F32 && dtype != ZO_BF16) return fail(ZO_ERR_UNSUPPORTED, "dtype %d", (int)dtype);
  if (n_heads < 1 || n_kv_heads < 1 || head_dim < 2)
    return fail(ZO_ERR_SHAPE, "n_heads = %d, n_kv_heads = %d, head_dim = %d", n_heads, n_kv_heads, head_dim);
  if (head_dim % 2 != 0 || head_dim > 256)
    return fail(ZO_ERR_UNSUPPORTED, "head_dim = %d: even values up to 256 are covered", head_dim);
  if ((gamma_q == nullptr) != (gamma_k == nullptr)) return fail(ZO_ERR_NULL, "gamma_q and gamma_k go together");
  if (!(norm_eps >= 0.0f)) return fail(ZO_ERR_SHAPE, "norm_eps = %g", (double)norm_eps);
  if ((int64_t)n_heads * head_dim > kMaxLd) return fail(ZO_ERR_SHAPE, "n_heads * head_dim too large");
  if (batch->n_tokens == 0) return ZO_OK;
  if (!Q || !K) return fail(ZO_ERR_NULL, "Q or K is NULL");
  if (int32_t st = check_matrix("Q", Q, ldq, n_heads * head_dim, dtype)) return st;
  if (int32_t st = check_matrix("K", K, ldk, n_kv_heads * head_dim, dtype)) return st;
  zo::QkRopeArgs a;
  a.Q = Q; a.ldq = ldq; a.K = K; a.ldk = ldk; a.cu = batch->cu_seqlens; a.S = batch->n_seqs; a.T = batch->n_tokens;
  a.n_heads = n_heads; a.n_kv_heads = n_kv_heads; a.dh = head_dim; a.gamma_q = gamma_q; a.gamma_k = gamma_k;
  a.eps = norm_eps; a.theta = rope_theta > 0.0f ? rope_theta : 0.0f; a.bf16 = dtype == ZO_BF16;
  ZO_HIP(zo::launch_qk_norm_rope(a, (hipStream_t)stream), "zo_qk_norm_rope");
  return ZO_OK;
}

}  // extern "C"
