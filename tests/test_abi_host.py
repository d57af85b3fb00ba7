"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/zo.h declares, its workspace queries are pure functions of
the shapes, and every argument error is reported before any device work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_28760_amd import binding as zb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000   # a non-NULL, 4 KiB aligned "device pointer" that is never dereferenced


def _declared():
    text = open(os.path.join(ROOT, "include", "zo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zo_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(names) == set(zb.EXPORTS)
    handle = zb.lib()
    for n in names:
        assert getattr(handle, n) is not None
    assert zb.zo_version() >= 1000


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(zb, "_lib", None)
    monkeypatch.setattr(zb, "LIB_PATH", "/nonexistent/libzo.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        zb.lib()


def _host_batch(lens=(3, 2), seq_cand=(0, 1), cand_dir=(0, 0), K=1, mirrors=True, T=None):
    cu = np.zeros(len(lens) + 1, np.int32); cu[1:] = np.cumsum(lens)
    sc = np.array(seq_cand, np.int32); cd = np.array(cand_dir, np.int32)
    return zb.make_batch(int(cu[-1]) if T is None else T, FAKE, FAKE, FAKE, FAKE, FAKE,
                         cu if mirrors else None, sc if mirrors else None, cd if mirrors else None,
                         n_seqs=len(lens), n_cands=len(cand_dir), n_dirs=K)


def _probe(batch, m=64, n=64, r=4, dt=zb.ZO_BF16, odt=None, X=FAKE, W=FAKE, Y=FAKE, ld=None, bank=None, act=0,
           ws=FAKE, ws_bytes=1 << 30):
    ld = n if ld is None else ld
    zb.zo_probe_linear(batch, X, ld, W, ld, None, m, n, dt, r, 1e-3, 0, bank, act, Y, m,
                       dt if odt is None else odt, ws, ws_bytes)


def _status(fn, *a, **k):
    with pytest.raises(zb.ZoError) as e:
        fn(*a, **k)
    return e.value.status


def test_batch_validation():
    assert _status(_probe, _host_batch(T=-1)) == zb.ZO_ERR_SHAPE
    b = _host_batch(); b.cu_seqlens = None
    assert _status(_probe, b) == zb.ZO_ERR_NULL
    b = _host_batch(); b.dir_seed = None
    assert _status(_probe, b) == zb.ZO_ERR_NULL
    assert _status(_probe, _host_batch(T=6)) == zb.ZO_ERR_INDEX                  # cu[S] != T
    bad = _host_batch(); np.frombuffer((C.c_int32 * 3).from_address(bad.host_cu_seqlens), np.int32)[:] = [0, 4, 3]
    assert _status(_probe, bad) == zb.ZO_ERR_INDEX                               # decreasing offsets
    assert _status(_probe, _host_batch(seq_cand=(0, 2))) == zb.ZO_ERR_INDEX      # candidate id >= C
    assert _status(_probe, _host_batch(seq_cand=(0, -2))) == zb.ZO_ERR_INDEX
    assert _status(_probe, _host_batch(cand_dir=(0, 1))) == zb.ZO_ERR_INDEX      # direction id >= K
    assert "cand_dir" in zb.last_error()


def test_probe_linear_validation():
    b = _host_batch()
    assert _status(_probe, b, r=0) == zb.ZO_ERR_SHAPE
    assert _status(_probe, b, r=513) == zb.ZO_ERR_SHAPE
    assert _status(_probe, b, X=None) == zb.ZO_ERR_NULL
    assert _status(_probe, b, n=72) == zb.ZO_ERR_UNSUPPORTED                     # bf16 needs n % 64 == 0
    assert _status(_probe, b, ld=60) == zb.ZO_ERR_SHAPE                          # ld < n
    assert _status(_probe, b, n=64, ld=68) == zb.ZO_ERR_SHAPE                    # rows not 16-byte aligned
    assert _status(_probe, b, X=FAKE + 2) == zb.ZO_ERR_SHAPE
    assert _status(_probe, b, dt=zb.ZO_F32, odt=zb.ZO_BF16) == zb.ZO_ERR_UNSUPPORTED
    assert _status(_probe, b, dt=5) == zb.ZO_ERR_UNSUPPORTED
    assert _status(_probe, b, act=3) == zb.ZO_ERR_UNSUPPORTED
    assert _status(_probe, b, act=2, m=63, dt=zb.ZO_F32) == zb.ZO_ERR_SHAPE            # (gate, up) pairs need an even m
    assert _status(_probe, b, act=2, m=24) == zb.ZO_ERR_UNSUPPORTED                    # 12 bf16 output columns
    assert _status(_probe, b, ws=None) == zb.ZO_ERR_WORKSPACE
    assert _status(_probe, b, ws=FAKE + 16) == zb.ZO_ERR_WORKSPACE
    assert _status(_probe, b, ws_bytes=16) == zb.ZO_ERR_WORKSPACE
    assert "needed" in zb.last_error()
    assert _status(_probe, b, bank=zb.make_bank(8, 9, FAKE, FAKE)) == zb.ZO_ERR_SHAPE
    assert _status(_probe, b, bank=zb.make_bank(8, 8, None, FAKE)) == zb.ZO_ERR_NULL
    # empty batch: nothing to do, no device work, success
    zb.zo_probe_linear(_host_batch(lens=(), seq_cand=(), cand_dir=(), K=0), None, 64, None, 64, None, 64, 64,
                       zb.ZO_BF16, 4, 1e-3, 0, None, 0, None, 64, zb.ZO_BF16, None, 0)


def test_workspace_queries_are_pure_and_monotone():
    q = zb.zo_probe_linear_workspace_bytes
    a = q(8192, 32, 1, 5120, 5120, 8, 64, zb.ZO_BF16)
    assert a == q(8192, 32, 1, 5120, 5120, 8, 64, zb.ZO_BF16) and a % 256 == 0
    assert q(8192, 32, 1, 5120, 5120, 8, 128, zb.ZO_BF16) > a
    assert q(16384, 32, 1, 5120, 5120, 8, 64, zb.ZO_BF16) > a
    assert q(0, 0, 0, 0, 0, 0, 0, zb.ZO_BF16) < 4096
    s = zb.zo_score_workspace_bytes(16384, 128, 50272, 5120, zb.ZO_BF16)
    assert s >= 2 * 197 * 16384 * 4 and s % 256 == 0
    assert zb.zo_score_workspace_bytes(16384, 128, 50272, 5120, zb.ZO_F32) > s   # narrower vocabulary tiles


def test_score_estimate_validation():
    b = _host_batch()
    sc = lambda **k: zb.zo_score(b, k.get("H", FAKE), k.get("ld", 64), FAKE, k.get("ld", 64), k.get("vocab", 100),
                                 k.get("d", 64), k.get("dt", zb.ZO_BF16), k.get("tg", FAKE), None, k.get("seq", FAKE),
                                 FAKE, FAKE, k.get("ws", FAKE), k.get("wsb", 1 << 30))
    assert _status(sc, vocab=0) == zb.ZO_ERR_SHAPE
    assert _status(sc, d=96, ld=96) == zb.ZO_ERR_UNSUPPORTED
    assert _status(sc, H=None) == zb.ZO_ERR_NULL
    assert _status(sc, tg=None) == zb.ZO_ERR_NULL
    assert _status(sc, seq=None) == zb.ZO_ERR_NULL
    assert _status(sc, wsb=8) == zb.ZO_ERR_WORKSPACE
    assert _status(zb.zo_estimate, b, FAKE, FAKE, 0.0, 0, FAKE, FAKE) == zb.ZO_ERR_SHAPE
    assert _status(zb.zo_estimate, b, FAKE, FAKE, 1e-3, 2, FAKE, FAKE) == zb.ZO_ERR_UNSUPPORTED
    assert _status(zb.zo_estimate, b, None, FAKE, 1e-3, 0, FAKE, FAKE) == zb.ZO_ERR_NULL


def test_bank_update_validation():
    col = lambda *v: np.array(v, np.int32)
    upd = lambda bank, c0, r=4, K=2, append=0, **k: zb.zo_bank_update(
        bank, 64, 64, r, K, k.get("seed", FAKE), 0, FAKE, 1e-3, None, c0, append, k.get("dt", zb.ZO_BF16))
    full = zb.make_bank(8, 8, FAKE, FAKE)
    assert _status(upd, full, col(0, 6)) == zb.ZO_ERR_BANK_FULL
    assert "R_cap" in zb.last_error()
    assert _status(upd, full, col(0, 2)) == zb.ZO_ERR_SHAPE                      # overlapping blocks
    assert _status(upd, full, col(-1, 4)) == zb.ZO_ERR_SHAPE
    assert _status(upd, zb.make_bank(8, 4, FAKE, FAKE), col(0, 4)) == zb.ZO_ERR_SHAPE   # accumulate beyond R_used
    assert _status(upd, full, col(0, 4), r=0) == zb.ZO_ERR_SHAPE
    assert _status(upd, full, col(0, 4), seed=None) == zb.ZO_ERR_NULL
    assert _status(upd, full, None) == zb.ZO_ERR_NULL
    assert _status(upd, zb.make_bank(8, 0, FAKE, None), col(0, 4), append=1) == zb.ZO_ERR_NULL
    assert _status(upd, full, col(0, 4), dt=3) == zb.ZO_ERR_UNSUPPORTED
    assert _status(lambda: zb.zo_factor_fill(1, 0, 4, 0, zb.ZO_F32, FAKE)) == zb.ZO_ERR_SHAPE
    assert _status(lambda: zb.zo_philox_words(1, 0, 0, -1, FAKE)) == zb.ZO_ERR_SHAPE
    assert _status(lambda: zb.zo_philox_words(1, 0, 0, 4, None)) == zb.ZO_ERR_NULL


def test_schedule_and_scheduled_update_validation():
    step = lambda **k: zb.zo_schedule_step(k.get("sched", FAKE), k.get("nu", 2), k.get("B", 2), k.get("K", 2), 1, 2,
                                           k.get("su", FAKE), k.get("sv", FAKE))
    assert _status(step, sched=None) == zb.ZO_ERR_NULL
    assert _status(step, nu=0) == zb.ZO_ERR_SHAPE
    assert _status(step, B=0) == zb.ZO_ERR_SHAPE
    assert _status(step, sv=None) == zb.ZO_ERR_NULL
    upd = lambda bank, **k: zb.zo_bank_update_scheduled(bank, 64, 64, k.get("r", 4), k.get("K", 2), FAKE, FAKE, 0, FAKE,
                                                        1e-3, None, k.get("sched", FAKE), k.get("B", 2), zb.ZO_BF16)
    assert _status(upd, zb.make_bank(8, 8, FAKE, FAKE)) == zb.ZO_ERR_BANK_FULL        # 2 blocks x 2 dirs x 4 > 8
    assert _status(upd, zb.make_bank(16, 8, FAKE, FAKE)) == zb.ZO_ERR_SHAPE          # blocks beyond R_used
    assert _status(upd, zb.make_bank(16, 16, FAKE, FAKE), sched=None) == zb.ZO_ERR_NULL
    assert _status(upd, zb.make_bank(16, 16, FAKE, None)) == zb.ZO_ERR_NULL
    assert _status(upd, zb.make_bank(16, 16, FAKE, FAKE), B=0) == zb.ZO_ERR_SHAPE
    assert C.sizeof(zb.zo_sched) == 32 and C.sizeof(zb.zo_batch) == 96


def test_fold_bank_validation():
    fold = lambda bank, **k: zb.zo_fold_bank(bank, k.get("W", FAKE), k.get("ld", 64), k.get("m", 64), k.get("n", 64),
                                             k.get("dt", zb.ZO_BF16))
    full = zb.make_bank(8, 8, FAKE, FAKE)
    assert _status(fold, full, W=None) == zb.ZO_ERR_NULL
    assert _status(fold, zb.make_bank(8, 8, FAKE, None)) == zb.ZO_ERR_NULL
    assert _status(fold, full, ld=32) == zb.ZO_ERR_SHAPE
    assert _status(fold, full, W=FAKE + 1) == zb.ZO_ERR_SHAPE
    assert _status(fold, full, dt=5) == zb.ZO_ERR_UNSUPPORTED
    assert _status(fold, zb.make_bank(8, 9, FAKE, FAKE)) == zb.ZO_ERR_SHAPE
    fold(zb.make_bank(8, 0, None, None), W=None)          # an empty bank folds to nothing, without device work


def test_add_norm_validation():
    def norm(**k):
        zb.zo_add_norm(k.get("X", FAKE), k.get("ldx", 64), k.get("R", FAKE), k.get("ldr", 64), k.get("gamma", FAKE),
                       k.get("beta", None), k.get("kind", zb.ZO_RMS_NORM), k.get("eps", 1e-6), k.get("T", 4),
                       k.get("d", 64), k.get("dt", zb.ZO_BF16), k.get("H", FAKE), k.get("ldh", 64), k.get("Y", FAKE),
                       k.get("ldy", 64))
    assert _status(norm, X=None) == zb.ZO_ERR_NULL
    assert _status(norm, H=None, Y=None) == zb.ZO_ERR_NULL          # nothing to compute
    assert _status(norm, R=None) == zb.ZO_ERR_NULL                  # a sum output without a residual
    assert _status(norm, gamma=None) == zb.ZO_ERR_NULL
    assert _status(norm, kind=2) == zb.ZO_ERR_UNSUPPORTED
    assert _status(norm, dt=4) == zb.ZO_ERR_UNSUPPORTED
    assert _status(norm, ldy=63) == zb.ZO_ERR_SHAPE
    assert _status(norm, ldr=8) == zb.ZO_ERR_SHAPE
    assert _status(norm, X=FAKE + 1) == zb.ZO_ERR_SHAPE
    assert _status(norm, Y=FAKE + 2, dt=zb.ZO_F32) == zb.ZO_ERR_SHAPE
    assert _status(norm, T=-1) == zb.ZO_ERR_SHAPE
    assert _status(norm, eps=-1.0) == zb.ZO_ERR_SHAPE
    norm(T=0, X=None)                                               # no rows: nothing is touched
    norm(d=0, X=None)


def test_attention_validation():
    def att(batch=None, **k):
        zb.zo_attention(batch or _host_batch(), k.get("Q", FAKE), k.get("ldq", 512), k.get("K", FAKE),
                        k.get("ldk", 512), k.get("V", FAKE), k.get("ldv", 512), k.get("H", 4), k.get("Hkv", 2),
                        k.get("dh", 128), 0.1, k.get("dt", zb.ZO_BF16), k.get("O", FAKE), k.get("ldo", 512))
    assert _status(att, Q=None) == zb.ZO_ERR_NULL
    assert _status(att, O=None) == zb.ZO_ERR_NULL
    assert _status(att, H=3) == zb.ZO_ERR_SHAPE                     # not a multiple of the key/value heads
    assert _status(att, H=0) == zb.ZO_ERR_SHAPE
    assert _status(att, dh=64) == zb.ZO_ERR_UNSUPPORTED             # the bf16 kernel is built for 128
    assert "head_dim" in zb.last_error()
    assert _status(att, dh=512, dt=zb.ZO_F32, ldq=4096, ldk=4096, ldv=4096, ldo=4096) == zb.ZO_ERR_UNSUPPORTED
    assert _status(att, ldq=256) == zb.ZO_ERR_SHAPE
    assert _status(att, ldk=128) == zb.ZO_ERR_SHAPE
    assert _status(att, ldo=516) == zb.ZO_ERR_SHAPE                 # rows would lose 16-byte alignment
    assert _status(att, V=FAKE + 2) == zb.ZO_ERR_SHAPE
    assert _status(att, dt=7) == zb.ZO_ERR_UNSUPPORTED
    assert _status(att, _host_batch(lens=(3, 2), T=6)) == zb.ZO_ERR_INDEX
    att(_host_batch(lens=(0, 0)), Q=None, O=None)                   # an empty batch needs no buffers


def test_qk_norm_rope_validation():
    def rope(batch=None, **k):
        zb.zo_qk_norm_rope(batch or _host_batch(), k.get("Q", FAKE), k.get("ldq", 512), k.get("K", FAKE),
                           k.get("ldk", 512), k.get("H", 4), k.get("Hkv", 2), k.get("dh", 128), k.get("gq", FAKE),
                           k.get("gk", FAKE), k.get("eps", 1e-6), 1e6, k.get("dt", zb.ZO_BF16))
    assert _status(rope, Q=None) == zb.ZO_ERR_NULL
    assert _status(rope, gk=None) == zb.ZO_ERR_NULL                 # the two gains go together
    assert _status(rope, dh=127) == zb.ZO_ERR_UNSUPPORTED
    assert _status(rope, dh=512, ldq=4096, ldk=4096) == zb.ZO_ERR_UNSUPPORTED
    assert _status(rope, H=0) == zb.ZO_ERR_SHAPE
    assert _status(rope, ldk=128) == zb.ZO_ERR_SHAPE
    assert _status(rope, eps=-1.0) == zb.ZO_ERR_SHAPE
    assert _status(rope, dt=9) == zb.ZO_ERR_UNSUPPORTED
    rope(_host_batch(lens=(0, 0)), Q=None, K=None)


def test_bank_update_multi_validation():
    def upd(entries, **k):
        arr = zb.make_layer_banks(entries)
        zb.zo_bank_update_multi(arr, k.get("r", 4), k.get("K", 1), k.get("seed", FAKE), None, FAKE, 1e-3, None,
                                np.array(k.get("col0", [0]), np.int32), k.get("append", 0), k.get("dt", zb.ZO_BF16))
        return arr
    good = (zb.make_bank(8, 8, FAKE, FAKE), 64, 64, 0)
    assert _status(upd, [good, (zb.make_bank(8, 8, None, FAKE), 64, 64, 2)]) == zb.ZO_ERR_NULL
    assert "layer 1" in zb.last_error()
    assert _status(upd, [good, (zb.make_bank(8, 2, FAKE, FAKE), 64, 64, 2)]) == zb.ZO_ERR_SHAPE      # beyond R_used
    assert _status(upd, [good], col0=[6]) == zb.ZO_ERR_BANK_FULL
    assert _status(upd, [good], r=0) == zb.ZO_ERR_SHAPE
    assert _status(upd, [good], seed=None) == zb.ZO_ERR_NULL
    assert _status(upd, [good], append=2) == zb.ZO_ERR_UNSUPPORTED
    assert _status(upd, [good, (zb.make_bank(8, 8, FAKE, FAKE), -1, 64, 2)]) == zb.ZO_ERR_SHAPE
    upd([])                                             # no layers: nothing to do
    upd([good], K=0, col0=[])                           # no directions either
    assert C.sizeof(zb.zo_layer_bank) == 40
