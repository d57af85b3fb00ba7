// Stand-ins for the kernel launchers and the three HIP calls that the host side of the C ABI
// (csrc/zo_abi.cpp) refers to, for a CPU-only build of that file under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Nothing is launched: a stub counts its calls and checks that every
// scratch pointer it is handed lies inside the workspace the test passed to the entry point.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "zo_internal.hpp"

int g_launches = 0;
const char* g_ws_lo = nullptr;
const char* g_ws_hi = nullptr;

static void inside(const void* p, size_t bytes, const char* what) {
  if (!p && bytes == 0) return;
  const char* c = (const char*)p;
  if (!g_ws_lo) return;
  if (c < g_ws_lo || c + bytes > g_ws_hi) {
    fprintf(stderr, "stub: %s [%p, +%zu) outside the workspace [%p, %p)\n", what, p, bytes, (const void*)g_ws_lo, (const void*)g_ws_hi);
    abort();
  }
}

extern "C" {
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
}

namespace zo {

int compute_units() { return 256; }
int head_vocab_tiles_bf16(int vocab) { return (vocab + kTileM - 1) / kTileM; }
int head_vocab_tiles_f32(int vocab) { return (vocab + kSimtTile - 1) / kSimtTile; }
int attention_f32_max_head_dim() { return 256; }
int attention_bf16_head_dim() { return 128; }

#define STUB(decl) hipError_t decl { ++g_launches; return hipSuccess; }
STUB(launch_philox_words(uint64_t, uint32_t, uint64_t, int64_t, uint32_t*, hipStream_t))
STUB(launch_factor_fill(uint64_t, uint32_t, int64_t, int, int, void*, hipStream_t))
STUB(launch_tok_index(const BatchDev&, int32_t*, int32_t*, hipStream_t))
STUB(launch_factors_f32(const BatchDev&, uint32_t, int, int, int, float*, float*, hipStream_t))
STUB(launch_probe_f32(const ProbeF32Args&, hipStream_t))
STUB(launch_head_score_f32(const HeadScoreF32Args&, hipStream_t))
STUB(launch_active_rows(const int32_t*, int, int32_t*, int32_t*, int32_t*, hipStream_t))
STUB(launch_estimate(const BatchDev&, const float*, const int32_t*, float, int, float*, float*, hipStream_t))
STUB(launch_estimate_es(const BatchDev&, const float*, const int32_t*, float, int, float*, float*, hipStream_t))
STUB(launch_schedule_step(SchedDev*, int, int, int, uint64_t, uint64_t, uint64_t*, uint64_t*, hipStream_t))
STUB(launch_bank_update(const BankUpdateArgs&, int, const int32_t*, hipStream_t))
STUB(launch_bank_update_multi(const BankUpdateArgs&, const BankLayer*, int, int, const int32_t*, hipStream_t))
STUB(launch_fold_bank(const FoldArgs&, hipStream_t))
STUB(launch_add_norm(const NormArgs&, hipStream_t))
STUB(launch_qk_norm_rope(const QkRopeArgs&, hipStream_t))
STUB(launch_attention(const AttnArgs&, hipStream_t))

hipError_t launch_seq_tables(const BatchDev& b, float, const SeqTables& t, hipStream_t) {
  ++g_launches;
  inside(t.seq_kind, (size_t)b.S * 4, "seq_kind");
  inside(t.seq_scale, (size_t)b.S * 4, "seq_scale");
  inside(t.tok_seq, (size_t)b.T * 4, "tok_seq");
  inside(t.items, (size_t)t.max_items * sizeof(SideItem), "items");
  inside(t.n_items, 8, "n_items");
  return hipSuccess;
}

hipError_t launch_probe_prep_bf16(const BatchDev& b, float eps, const SeqTables& t, uint32_t, int, int n, int, int RP,
                                  int Rp, const float*, const float*, int, int, int m_img, uint16_t* Uimg, uint16_t* Vt,
                                  uint16_t* Pimg, uint16_t* Vbt, hipStream_t st) {
  launch_seq_tables(b, eps, t, st);
  inside(t.tile_hdr, (size_t)t.n_tn * sizeof(TileHdr), "tile_hdr");
  inside(t.tile_slots, (size_t)t.slot_cap * 4, "tile_slots");
  inside(t.kt_tile, (size_t)t.kt_cap * 4, "kt_tile");
  inside(Uimg, (size_t)b.K * t.SPD * m_img * 64, "Uimg");
  inside(Pimg, (size_t)t.RpT * m_img * 128, "Pimg");
  inside(Vt, (size_t)b.K * RP * n * 2, "Vt");
  inside(Vbt, (size_t)Rp * n * 2, "Vbt");
  return hipSuccess;
}

hipError_t launch_side_down_bf16(const SideDownArgs& a, hipStream_t) {
  ++g_launches;
  inside(a.partial, (size_t)a.ksplit * a.T * (a.RP + a.Rp) * 4, "partial");
  inside(a.Xs, (size_t)a.kt_cap * kTileN * kTileK * 2, "Xs");
  if (a.ksplit < 1 || a.ksplit > 8 || (a.item_rows != 16 && a.item_rows != 32 && a.item_rows != 48 && a.item_rows != 64)) abort();
  return hipSuccess;
}

hipError_t launch_probe_gemm_bf16(const ProbeGemmArgs& a, hipStream_t) {
  ++g_launches;
  if (a.has_side) {
    inside(a.Uimg, (size_t)a.uimg_bytes, "Uimg (GEMM)");
    inside(a.Pimg, (size_t)a.pimg_bytes, "Pimg (GEMM)");
    inside(a.Xs, (size_t)a.xs_bytes, "Xs (GEMM)");
  }
  return hipSuccess;
}

hipError_t launch_head_score_bf16(const HeadScoreArgs& a, hipStream_t) {
  ++g_launches;
  const size_t n_vt = (size_t)head_vocab_tiles_bf16(a.vocab);
  inside(a.part_max, n_vt * a.T * 4, "part_max");
  inside(a.part_sum, n_vt * a.T * 4, "part_sum");
  inside(a.tgt_logit, (size_t)a.T * 4, "tgt_logit");
  if (a.rows) inside(a.rows, (size_t)a.T * 4, "rows");
  return hipSuccess;
}

hipError_t launch_score_combine(const ScoreCombineArgs& a, hipStream_t) {
  ++g_launches;
  inside(a.seq_cnt, (size_t)a.S * 4, "seq_cnt");
  return hipSuccess;
}

}  // namespace zo
