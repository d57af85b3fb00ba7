// Drives the host side of the C ABI (argument validation, workspace planning, call sequencing) in a
// CPU-only build under AddressSanitizer and UndefinedBehaviorSanitizer: every error class of every entry
// point once, then valid calls of the planning paths at the sizes of the benchmark configurations, whose
// scratch pointers the stub launchers check against the workspace.  Device pointers are fake addresses
// that nothing dereferences.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/zo.h"

extern int g_launches;
extern const char* g_ws_lo;
extern const char* g_ws_hi;

static int g_checks = 0, g_failed = 0;
#define EXPECT(call, want)                                                                    \
  do {                                                                                        \
    const int32_t got__ = (call);                                                             \
    ++g_checks;                                                                               \
    if (got__ != (want)) {                                                                    \
      char msg[512];                                                                          \
      zo_last_error(msg, sizeof msg);                                                         \
      fprintf(stderr, "line %d: %s -> %d, expected %d (%s)\n", __LINE__, #call, got__, (int)(want), msg); \
      ++g_failed;                                                                             \
    }                                                                                         \
  } while (0)

static void* const FAKE = (void*)(uintptr_t)0x7f0000000000ull;   // a 256-byte aligned "device" address

struct HostBatch {
  std::vector<int32_t> cu, seq_cand, cand_dir;
  zo_batch b;
};

static HostBatch make_batch(int T, std::vector<int32_t> cu, std::vector<int32_t> seq_cand, std::vector<int32_t> cand_dir,
                            int K) {
  HostBatch h;
  h.cu = cu; h.seq_cand = seq_cand; h.cand_dir = cand_dir;
  memset(&h.b, 0, sizeof h.b);
  h.b.n_tokens = T; h.b.n_seqs = (int)seq_cand.size(); h.b.n_cands = (int)cand_dir.size(); h.b.n_dirs = K;
  h.b.cu_seqlens = (const int32_t*)FAKE; h.b.seq_cand = (const int32_t*)FAKE; h.b.cand_dir = (const int32_t*)FAKE;
  h.b.cand_sign = (const float*)FAKE; h.b.dir_seed = (const uint64_t*)FAKE;
  return h;
}
static void mirror(HostBatch& h) {
  h.b.host_cu_seqlens = h.cu.data(); h.b.host_seq_cand = h.seq_cand.data(); h.b.host_cand_dir = h.cand_dir.data();
}

static int32_t probe(const zo_batch* b, const void* X, int64_t ld, int m, int n, zo_dtype dt, int r, const zo_bank* bank,
                     int act, zo_dtype odt, void* ws, size_t wsb) {
  return zo_probe_linear(b, X, ld, FAKE, ld, nullptr, m, n, dt, r, 1e-3f, 0, bank, act, FAKE, m, odt, ws, wsb, nullptr);
}

int main() {
  // ---- batch validation ----------------------------------------------------------------------
  {
    HostBatch h = make_batch(8, {0, 4, 8}, {0, 1}, {0, 0}, 1);
    mirror(h);
    const size_t wsb = zo_probe_linear_workspace_bytes(8, 2, 1, 64, 64, 4, 0, ZO_BF16);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_OK);
    EXPECT(probe(nullptr, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_NULL);
    HostBatch neg = h; neg.b.n_tokens = -1;
    EXPECT(probe(&neg.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    HostBatch nocu = h; nocu.b.cu_seqlens = nullptr;
    EXPECT(probe(&nocu.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_NULL);
    HostBatch badT = make_batch(6, {0, 4, 8}, {0, 1}, {0, 0}, 1); mirror(badT);
    EXPECT(probe(&badT.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_INDEX);
    HostBatch dec = make_batch(8, {0, 9, 8}, {0, 1}, {0, 0}, 1); mirror(dec);
    EXPECT(probe(&dec.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_INDEX);
    HostBatch badc = make_batch(8, {0, 4, 8}, {0, 2}, {0, 0}, 1); mirror(badc);
    EXPECT(probe(&badc.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_INDEX);
    HostBatch badd = make_batch(8, {0, 4, 8}, {0, 1}, {0, 1}, 1); mirror(badd);
    EXPECT(probe(&badd.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_INDEX);

    // ---- probe linear -------------------------------------------------------------------------
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 0, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 513, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    EXPECT(probe(&h.b, nullptr, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_NULL);
    EXPECT(probe(&h.b, FAKE, 72, 64, 72, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_UNSUPPORTED);
    EXPECT(probe(&h.b, FAKE, 60, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    EXPECT(probe(&h.b, (char*)FAKE + 2, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_F32, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_UNSUPPORTED);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, (zo_dtype)5, 4, nullptr, 0, ZO_BF16, FAKE, wsb), ZO_ERR_UNSUPPORTED);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 3, ZO_BF16, FAKE, wsb), ZO_ERR_UNSUPPORTED);
    EXPECT(probe(&h.b, FAKE, 64, 63, 64, ZO_F32, 4, nullptr, 2, ZO_F32, FAKE, wsb), ZO_ERR_SHAPE);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, nullptr, wsb), ZO_ERR_WORKSPACE);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, (char*)FAKE + 16, wsb), ZO_ERR_WORKSPACE);
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, nullptr, 0, ZO_BF16, FAKE, 16), ZO_ERR_WORKSPACE);
    zo_bank over = {8, 9, (float*)FAKE, (float*)FAKE};
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, &over, 0, ZO_BF16, FAKE, wsb), ZO_ERR_SHAPE);
    zo_bank nop = {8, 8, nullptr, (float*)FAKE};
    EXPECT(probe(&h.b, FAKE, 64, 64, 64, ZO_BF16, 4, &nop, 0, ZO_BF16, FAKE, wsb), ZO_ERR_NULL);

    // ---- scoring, estimate --------------------------------------------------------------------
    const size_t ssb = zo_score_workspace_bytes(8, 2, 100, 64, ZO_BF16);
    auto score = [&](const void* H, int vocab, int d, const int32_t* tg, float* seq, size_t bytes) {
      return zo_score(&h.b, H, d, FAKE, d, vocab, d, ZO_BF16, tg, nullptr, seq, (float*)FAKE, (int32_t*)FAKE, FAKE, bytes, nullptr);
    };
    EXPECT(score(FAKE, 100, 64, (const int32_t*)FAKE, (float*)FAKE, ssb), ZO_OK);
    EXPECT(score(FAKE, 0, 64, (const int32_t*)FAKE, (float*)FAKE, ssb), ZO_ERR_SHAPE);
    EXPECT(score(FAKE, 100, 96, (const int32_t*)FAKE, (float*)FAKE, ssb), ZO_ERR_UNSUPPORTED);
    EXPECT(score(nullptr, 100, 64, (const int32_t*)FAKE, (float*)FAKE, ssb), ZO_ERR_NULL);
    EXPECT(score(FAKE, 100, 64, nullptr, (float*)FAKE, ssb), ZO_ERR_NULL);
    EXPECT(score(FAKE, 100, 64, (const int32_t*)FAKE, nullptr, ssb), ZO_ERR_NULL);
    EXPECT(score(FAKE, 100, 64, (const int32_t*)FAKE, (float*)FAKE, 8), ZO_ERR_WORKSPACE);
    EXPECT(zo_estimate(&h.b, (float*)FAKE, (int32_t*)FAKE, 0.0f, 0, (float*)FAKE, (float*)FAKE, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_estimate(&h.b, (float*)FAKE, (int32_t*)FAKE, 1e-3f, 2, (float*)FAKE, (float*)FAKE, nullptr), ZO_ERR_UNSUPPORTED);
    EXPECT(zo_estimate(&h.b, nullptr, (int32_t*)FAKE, 1e-3f, 0, (float*)FAKE, (float*)FAKE, nullptr), ZO_ERR_NULL);
    EXPECT(zo_estimate(&h.b, (float*)FAKE, (int32_t*)FAKE, 1e-3f, 0, (float*)FAKE, (float*)FAKE, nullptr), ZO_OK);
    EXPECT(zo_estimate_es(&h.b, (float*)FAKE, (int32_t*)FAKE, 1e-3f, 1, (float*)FAKE, (float*)FAKE, nullptr), ZO_OK);
  }
  // ---- bank update, schedule, fold ---------------------------------------------------------------
  {
    zo_bank full = {8, 8, (float*)FAKE, (float*)FAKE};
    const int32_t c04[2] = {0, 4}, c06[2] = {0, 6}, c02[2] = {0, 2}, cm1[2] = {-1, 4};
    auto upd = [&](zo_bank* b, const int32_t* col0, int r, const uint64_t* seed, int append, zo_dtype dt) {
      return zo_bank_update(b, 32, 32, r, 2, seed, nullptr, 0, (float*)FAKE, 1e-3f, nullptr, col0, append, dt, nullptr);
    };
    EXPECT(upd(&full, c04, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_OK);
    EXPECT(upd(&full, c06, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_BANK_FULL);
    EXPECT(upd(&full, c02, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_SHAPE);
    EXPECT(upd(&full, cm1, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_SHAPE);
    zo_bank half = {8, 4, (float*)FAKE, (float*)FAKE};
    EXPECT(upd(&half, c04, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_SHAPE);
    EXPECT(upd(&half, c04, 4, (uint64_t*)FAKE, 1, ZO_F32), ZO_OK);
    EXPECT(half.R_used == 8 ? 0 : 1, 0);
    EXPECT(upd(&full, c04, 0, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_SHAPE);
    EXPECT(upd(&full, c04, 4, nullptr, 0, ZO_F32), ZO_ERR_NULL);
    EXPECT(upd(&full, nullptr, 4, (uint64_t*)FAKE, 0, ZO_F32), ZO_ERR_NULL);
    EXPECT(upd(&full, c04, 4, (uint64_t*)FAKE, 0, (zo_dtype)3), ZO_ERR_UNSUPPORTED);
    zo_layer_bank layers[3];
    for (int i = 0; i < 3; ++i) { layers[i].bank = full; layers[i].m = 32 + i; layers[i].n = 16; layers[i].tensor_id = 2 * i; layers[i].reserved = 0; }
    EXPECT(zo_bank_update_multi(layers, 3, 4, 2, (uint64_t*)FAKE, nullptr, (float*)FAKE, 1e-3f, nullptr, c04, 0, ZO_BF16, nullptr), ZO_OK);
    EXPECT(zo_bank_update_multi(layers, 3, 4, 2, (uint64_t*)FAKE, nullptr, (float*)FAKE, 1e-3f, nullptr, c06, 0, ZO_BF16, nullptr), ZO_ERR_BANK_FULL);
    EXPECT(zo_bank_update_multi(nullptr, 3, 4, 2, (uint64_t*)FAKE, nullptr, (float*)FAKE, 1e-3f, nullptr, c04, 0, ZO_BF16, nullptr), ZO_ERR_NULL);
    EXPECT(zo_factor_fill(1, 0, 4, 0, ZO_F32, FAKE, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_philox_words(1, 0, 0, -1, (uint32_t*)FAKE, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_philox_words(1, 0, 0, 4, nullptr, nullptr), ZO_ERR_NULL);
    EXPECT(zo_schedule_step(nullptr, 2, 2, 2, 1, 2, (uint64_t*)FAKE, (uint64_t*)FAKE, nullptr), ZO_ERR_NULL);
    EXPECT(zo_schedule_step((zo_sched*)FAKE, 0, 2, 2, 1, 2, (uint64_t*)FAKE, (uint64_t*)FAKE, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_schedule_step((zo_sched*)FAKE, 2, 2, 2, 1, 2, (uint64_t*)FAKE, (uint64_t*)FAKE, nullptr), ZO_OK);
    zo_bank b16 = {16, 16, (float*)FAKE, (float*)FAKE};
    EXPECT(zo_bank_update_scheduled(&b16, 32, 32, 4, 2, (uint64_t*)FAKE, (uint64_t*)FAKE, 0, (float*)FAKE, 1e-3f, nullptr,
                                    (zo_sched*)FAKE, 2, ZO_F32, nullptr), ZO_OK);
    EXPECT(zo_bank_update_scheduled(&full, 32, 32, 4, 2, (uint64_t*)FAKE, (uint64_t*)FAKE, 0, (float*)FAKE, 1e-3f, nullptr,
                                    (zo_sched*)FAKE, 2, ZO_F32, nullptr), ZO_ERR_BANK_FULL);
    EXPECT(zo_fold_bank(&full, FAKE, 64, 32, 64, ZO_BF16, nullptr), ZO_OK);
    EXPECT(zo_fold_bank(&full, nullptr, 64, 32, 64, ZO_BF16, nullptr), ZO_ERR_NULL);
    EXPECT(zo_fold_bank(&full, FAKE, 32, 32, 64, ZO_BF16, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_fold_bank(&full, FAKE, 64, 32, 64, (zo_dtype)5, nullptr), ZO_ERR_UNSUPPORTED);
  }
  // ---- block entry points --------------------------------------------------------------------
  {
    HostBatch h = make_batch(8, {0, 4, 8}, {0, 1}, {0, 0}, 1);
    EXPECT(zo_add_norm(FAKE, 64, nullptr, 0, (float*)FAKE, nullptr, ZO_RMS_NORM, 1e-6f, 8, 64, ZO_BF16, nullptr, 0, FAKE, 64, nullptr), ZO_OK);
    EXPECT(zo_add_norm(FAKE, 64, nullptr, 0, (float*)FAKE, nullptr, 7, 1e-6f, 8, 64, ZO_BF16, nullptr, 0, FAKE, 64, nullptr), ZO_ERR_UNSUPPORTED);
    EXPECT(zo_add_norm(FAKE, 64, nullptr, 0, (float*)FAKE, nullptr, ZO_RMS_NORM, 1e-6f, 8, 64, ZO_BF16, nullptr, 0, nullptr, 64, nullptr), ZO_ERR_NULL);
    EXPECT(zo_attention(&h.b, FAKE, 512, FAKE, 512, FAKE, 512, 4, 2, 128, 0.1f, ZO_BF16, FAKE, 512, nullptr), ZO_OK);
    EXPECT(zo_attention(&h.b, FAKE, 512, FAKE, 512, FAKE, 512, 4, 3, 128, 0.1f, ZO_BF16, FAKE, 512, nullptr), ZO_ERR_SHAPE);
    EXPECT(zo_attention(&h.b, FAKE, 512, FAKE, 512, FAKE, 512, 4, 2, 64, 0.1f, ZO_BF16, FAKE, 512, nullptr), ZO_ERR_UNSUPPORTED);
    EXPECT(zo_qk_norm_rope(&h.b, FAKE, 512, FAKE, 256, 4, 2, 128, (float*)FAKE, (float*)FAKE, 1e-6f, 1e6f, ZO_BF16, nullptr), ZO_OK);
    EXPECT(zo_qk_norm_rope(&h.b, FAKE, 512, FAKE, 256, 4, 2, 128, (float*)FAKE, nullptr, 1e-6f, 1e6f, ZO_BF16, nullptr), ZO_ERR_NULL);
  }
  // ---- workspace planning at the benchmark sizes: every scratch region inside the workspace ---------
  {
    struct Case { int T, S, C, K, m, n, r, R, vocab; } cases[] = {
        {8192, 32, 2, 1, 5120, 5120, 8, 64, 0},        {8192, 32, 2, 1, 5120, 20480, 8, 64, 0},
        {16384, 128, 2, 1, 20480, 5120, 8, 64, 50272}, {19828, 64, 32, 16, 12288, 4096, 16, 128, 151936},
        {33451, 64, 48, 24, 4096, 12288, 16, 128, 151936}, {300, 300, 64, 64, 200, 128, 512, 300, 1187},
        {1, 1, 1, 1, 8, 64, 1, 0, 2},                  {70000, 3, 2, 1, 256, 64, 40, 160, 64}};
    for (const Case& c : cases) {
      std::vector<int32_t> cu(c.S + 1), sc(c.S), cd(c.C, 0);
      for (int s = 0; s <= c.S; ++s) cu[s] = (int32_t)((int64_t)c.T * s / c.S);
      for (int s = 0; s < c.S; ++s) sc[s] = s % c.C;
      for (int k = 0; k < c.C; ++k) cd[k] = k % c.K;
      HostBatch h = make_batch(c.T, cu, sc, cd, c.K);
      mirror(h);
      for (zo_dtype dt : {ZO_BF16, ZO_F32}) {
        const size_t wsb = zo_probe_linear_workspace_bytes(c.T, c.S, c.K, c.m, c.n, c.r, c.R, dt);
        g_ws_lo = (const char*)FAKE; g_ws_hi = g_ws_lo + wsb;
        zo_bank bank = {c.R, c.R, (float*)FAKE, (float*)FAKE};
        const int before = g_launches;
        EXPECT(zo_probe_linear(&h.b, FAKE, c.n, FAKE, c.n, nullptr, c.m, c.n, dt, c.r, 1e-3f, 4, c.R ? &bank : nullptr, 1, FAKE,
                               c.m, dt, FAKE, wsb, nullptr), ZO_OK);
        EXPECT(g_launches > before ? 0 : 1, 0);
        // a workspace sized for this batch also serves a smaller one
        HostBatch small = h; small.b.n_tokens = c.T / 2 + 1; small.b.host_cu_seqlens = nullptr;
        EXPECT(zo_probe_linear(&small.b, FAKE, c.n, FAKE, c.n, nullptr, c.m, c.n, dt, c.r, 1e-3f, 4, c.R ? &bank : nullptr, 1,
                               FAKE, c.m, dt, FAKE, wsb, nullptr), ZO_OK);
        if (c.vocab > 0) {
          const int d = c.m % 64 == 0 ? c.m : 64;
          const size_t ssb = zo_score_workspace_bytes(c.T, c.S, c.vocab, d, dt);
          g_ws_hi = g_ws_lo + ssb;
          EXPECT(zo_score(&h.b, FAKE, d, FAKE, d, c.vocab, d, dt, (int32_t*)FAKE, nullptr, (float*)FAKE, (float*)FAKE,
                          (int32_t*)FAKE, FAKE, ssb, nullptr), ZO_OK);
        }
        g_ws_lo = g_ws_hi = nullptr;
      }
    }
    EXPECT(zo_probe_linear_workspace_bytes(-1, 1, 1, 8, 64, 1, 0, ZO_BF16) == 0 ? 0 : 1, 0);
  }
  char msg[64];
  zo_last_error(msg, sizeof msg);   // short buffer: truncation path
  zo_last_error(nullptr, 0);
  printf("abi host check: %d checks, %d failed, %d stub launches\n", g_checks, g_failed, g_launches);
  return g_failed ? 1 : 0;
}
