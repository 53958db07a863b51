"""The C-ABI library loads and exports what include/guard.h declares; host-side
validation answers with status codes (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2605_17879_amd import guard

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "guard.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = guard.load_library()
    names = declared_symbols()
    assert set(names) == set(guard.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_header_is_plain_c(tmp_path):
    """include/guard.h is the boundary: it must compile as C99 and as C++ on its own."""
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "guard.h"\nint main(void) { gd_config c; gd_ledger_config l; (void)c; (void)l; return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(src),
                    "-o", str(tmp_path / "t.o")], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-I", inc, "-x", "c++", "-c", str(src),
                    "-o", str(tmp_path / "t2.o")], check=True)


def make(**kw):
    lib = guard.load_library()
    c = guard.Config(n_ranks=kw.pop("R", 64), n_metrics=kw.pop("M", 2), window=kw.pop("W", 8),
                     persist_k=kw.pop("k", 4), **kw).to_c()
    h = ctypes.c_void_p()
    st = lib.gd_create(ctypes.byref(c), ctypes.byref(h))
    return lib, st, h


def test_defaults():
    c = guard.Config(65536, 8, 256, 200).to_c()
    assert c.struct_size == ctypes.sizeof(guard._CConfig) == 64
    assert (c.gpus_per_node, c.primary_metric, c.min_signals, c.topk) == (8, 0, 2, 64)
    assert c.z_threshold == 3.5 and abs(c.node_scale - 8 ** -0.5) < 1e-7
    assert guard.Config(64, 1, 20, 15).to_c().min_signals == 1
    assert guard.Config(64, 1, 20, 15).to_c().topk == 8


@pytest.mark.parametrize("kw,status", [
    (dict(R=60), 2), (dict(R=0), 2), (dict(R=65544), 4), (dict(M=0), 2), (dict(M=9), 2),
    (dict(W=0), 2), (dict(W=1025), 2), (dict(k=9), 2), (dict(k=0), 2), (dict(primary_metric=2), 2),
    (dict(min_signals=3), 2), (dict(gpus_per_node=4), 4), (dict(topk=9), 2), (dict(node_agg=2), 2),
    (dict(abs_floor=0.0), 2), (dict(z_threshold=float("nan")), 2), (dict(direction=(2, 1)), 2),
])
def test_bad_configurations_are_refused(kw, status):
    lib, st, h = make(**kw)
    assert st == status and not h.value
    assert len(lib.gd_last_error(None)) > 0


def test_state_size_and_argument_checks_without_a_device():
    lib, st, h = make(R=1024, M=4, W=50, k=40)
    assert st == 0 and h.value
    n = lib.gd_state_bytes(h)
    # rings + counters + first-flag steps + latest node score, each 256-byte aligned
    want = 0
    for b in (50 * 16 * 8, 50 * 2 * 8, 1024 * 2, 128 * 2, 1024 * 4, 128 * 4, 128 * 4):
        want += (b + 255) // 256 * 256
    assert n == want
    # nothing bound yet / null pointers / misaligned: status codes, no launch
    assert lib.gd_update_window(h, 256, 256, 256, 1, 0, None) == 1
    assert lib.gd_flags(h, None, None, None, None, None, None, None) == 1
    assert lib.gd_topk_nodes(h, 4, 256, None, None) == 1
    assert lib.gd_severity(h, 256, 1, 256, 0.1, 0.2, 256, 256, None) == 1     # no state bound
    assert lib.gd_sweep_score(h, None, 256, 3, 0.05, 0.1, 0.15, 256, 256, 256, 256, None) == 1
    assert lib.gd_sweep_score(h, None, None, 0, 0.05, 0.1, 0.15, None, None, None, None, None) == 0
    assert lib.gd_probe_read(h, None, 1 << 20, 256, None) == 1
    assert lib.gd_apply_membership(h, None, 1, 256, None) == 1
    assert lib.gd_apply_membership(h, 256 + 4, 1, 256, None) == 1   # x not 16-byte aligned
    assert lib.gd_apply_membership(h, 256, 70000, 256, None) == 1
    assert lib.gd_apply_membership(h, None, 0, None, None) == 0
    assert lib.gd_set_streaming_hints(h, 256, None) == 1        # both or neither
    assert lib.gd_set_streaming_hints(h, 256 + 2, 256) == 1     # misaligned
    assert lib.gd_set_streaming_hints(h, 256, 512) == 0
    assert lib.gd_set_streaming_hints(h, None, None) == 0
    assert lib.gd_bind_state(h, None, n) == 1
    assert lib.gd_bind_state(h, 4096 + 8, n) == 1          # misaligned
    assert lib.gd_bind_state(h, 4096, n - 1) == 3          # too small
    assert lib.gd_score_batch(h, None, 1, *([256] * 8), None) == 1
    assert lib.gd_score_batch(h, 256 + 4, 1, *([256] * 8), None) == 1   # x not 16-byte aligned
    assert lib.gd_score_batch(h, None, 0, *([None] * 8), None) == 0     # T == 0: no-op
    assert b"null" in lib.gd_last_error(h) or b"align" in lib.gd_last_error(h)
    assert lib.gd_destroy(h) == 0


def test_ledger_size_and_argument_checks_without_a_device():
    lib, st, h = make(R=1024, M=4, W=50, k=40)
    assert st == 0
    c = guard._CLedgerConfig()
    lib.gd_default_ledger_config(ctypes.byref(c))
    assert c.struct_size == ctypes.sizeof(guard._CLedgerConfig) == 24
    assert (c.score_quant, c.recur_limit, c.recur_horizon) == (64.0, 3, 604800)
    up = lambda b: (b + 255) // 256 * 256
    counts = up(1024 * 16) + up(128 * 16) + up(128 * 2)
    want = (up(32) + up(50 * 1024) + up(50 * 128) + 2 * counts + up(1024 * 4) + up(128 * 4) +
            up(50 * 128 * 2) + up(128 * 4) + up(128 * 32) + up(128 * 4) + up(300 * 2 * 8))
    n = lib.gd_ledger_bytes(h, 300)
    assert n == want
    assert lib.gd_ledger_bytes(None, 300) == 0
    # nothing bound yet
    assert lib.gd_update_ledger(h, 256, 256, 256, 1, 0, None) == 1
    assert lib.gd_ledger_flags(h, *([None] * 10)) == 1
    assert lib.gd_topk_nodes_mean(h, 4, 256, None, None) == 1
    # binding: null, misaligned, too small, bad configurations
    assert lib.gd_bind_ledger(h, ctypes.byref(c), None, n, 300) == 1
    assert lib.gd_bind_ledger(h, None, 4096, n, 300) == 1
    assert lib.gd_bind_ledger(h, ctypes.byref(c), 4096 + 8, n, 300) == 1
    assert lib.gd_bind_ledger(h, ctypes.byref(c), 4096, n - 1, 300) == 3
    assert lib.gd_bind_ledger(h, ctypes.byref(c), 4096, n, 0) == 1
    for name, bad in (("score_quant", 0.0), ("score_quant", float("inf")), ("recur_limit", 0),
                      ("recur_limit", 9), ("recur_horizon", 0), ("struct_size", 8)):
        d = guard._CLedgerConfig()
        lib.gd_default_ledger_config(ctypes.byref(d))
        setattr(d, name, bad)
        assert lib.gd_bind_ledger(h, ctypes.byref(d), 4096, n, 300) == 2, name
    # bound (the address is never touched without a launch): argument checks of the update
    assert lib.gd_bind_ledger(h, ctypes.byref(c), 4096, n, 300) == 0
    assert lib.gd_update_ledger(h, None, None, None, 0, 0, None) == 0          # T == 0: no-op
    assert lib.gd_update_ledger(h, None, 256, 256, 1, 0, None) == 1
    assert lib.gd_update_ledger(h, 256, 256, 256, 301, 0, None) == 1           # more than max_T
    assert lib.gd_update_ledger(h, 256 + 1, 256, 256, 1, 0, None) == 1         # misaligned
    assert lib.gd_update_ledger(h, 256, 256, 256, 2, 2**31 - 2, None) == 1     # step index too large
    assert lib.gd_topk_nodes_mean(h, 129, 256, None, None) == 1
    assert lib.gd_topk_nodes_mean(h, 4, None, None, None) == 1
    assert lib.gd_destroy(h) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(guard, "_lib", None)
    monkeypatch.setattr(guard, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        guard.load_library()
