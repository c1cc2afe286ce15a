"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a GPU (CPU only)."""
import ctypes as C
import os
import re

import pytest

from paper_2010_16248_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2010_16248_amd import build
        build.build(verbose=False)
    return B.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "accordion.h")).read()
    declared = sorted(set(re.findall(r"\b(accordion_[a-z_]+)\s*\(", header)))
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == declared


def _cfg(**kw):
    layers = kw.pop("layers", [(0, 8, 12, 1), (96, 1, 10, 0)])
    args = dict(method=B.ACC_TOPK, layers=layers, n_workers=2, level_crit=10, level_noncrit=1)
    args.update(kw)
    return B.make_config(**args)


def test_workspace_bytes_is_host_arithmetic(lib):
    cfg, keep = _cfg()
    n = B.accordion_workspace_bytes(cfg)
    assert n > 0 and n % 256 == 0
    cfg2, keep2 = _cfg(n_workers=4)
    assert B.accordion_workspace_bytes(cfg2) > n
    cfgp, keepp = _cfg(method=B.ACC_POWERSGD, level_crit=4, level_noncrit=1)
    assert B.accordion_workspace_bytes(cfgp) > 0


@pytest.mark.parametrize("mutate,msg", [
    (lambda c: setattr(c, "n_workers", 0), "n_workers"),
    (lambda c: setattr(c, "n_workers", 33), "n_workers"),
    (lambda c: setattr(c, "n_layers", 0), "n_layers"),
    (lambda c: setattr(c, "method", 7), "method"),
    (lambda c: setattr(c, "k_num_crit", 101), "k fraction"),
    (lambda c: setattr(c, "k_den", 0), "k fraction"),
    (lambda c: setattr(c, "eta", float("nan")), "eta"),
    (lambda c: setattr(c, "initial_level", 2), "initial_level"),
    (lambda c: setattr(c, "n_params", 50), "outside"),
])
def test_invalid_configs_are_rejected(lib, mutate, msg):
    cfg, keep = _cfg()
    mutate(cfg)
    out = C.c_size_t(0)
    rc = lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out))
    assert rc == B.ACC_EINVAL
    assert msg in lib.accordion_last_error(None).decode()


def test_invalid_layers_and_ranks(lib):
    out = C.c_size_t(0)
    cfg, keep = _cfg(layers=[(0, 8, 12, 1), (90, 1, 10, 0)])          # overlap
    assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_EINVAL
    assert "overlap" in lib.accordion_last_error(None).decode()
    cfg, keep = _cfg(layers=[(0, 0, 12, 1)])
    assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_EINVAL
    cfg, keep = _cfg(method=B.ACC_POWERSGD, level_crit=5, level_noncrit=1)
    assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_EINVAL
    assert lib.accordion_workspace_bytes(None, C.byref(out)) == B.ACC_EINVAL
    cfg, keep = _cfg()
    assert lib.accordion_workspace_bytes(C.byref(cfg), None) == B.ACC_EINVAL


def test_batch_size_mode_config(lib):
    out = C.c_size_t(0)
    cfg, keep = _cfg(method=B.ACC_BATCH, batch_multiplier=8)
    assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_OK
    # W sums + accumulator + tables: far smaller than the TopK workspace of the same model
    cfgt, keept = _cfg()
    assert 0 < out.value < B.accordion_workspace_bytes(cfgt)
    for bad in (0, -1, 65537):
        cfg, keep = _cfg(method=B.ACC_BATCH, batch_multiplier=bad)
        assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_EINVAL
        assert "batch_multiplier" in lib.accordion_last_error(None).decode()
    cfg, keep = _cfg(method=B.ACC_BATCH, batch_multiplier=8, batch_monotone=2)
    assert lib.accordion_workspace_bytes(C.byref(cfg), C.byref(out)) == B.ACC_EINVAL
    assert lib.accordion_batch_status(None, None, None, None, None, None) == B.ACC_EINVAL


def test_init_rejects_null_and_small_workspace_without_a_gpu(lib):
    cfg, keep = _cfg()
    ctx = C.c_void_p(None)
    assert lib.accordion_init(C.byref(cfg), None, 1 << 30, None, None, C.byref(ctx)) == B.ACC_EINVAL
    assert ctx.value is None
    assert lib.accordion_init(C.byref(cfg), C.c_void_p(256), 16, None, None, C.byref(ctx)) == B.ACC_ENOSPACE
    assert lib.accordion_init(C.byref(cfg), C.c_void_p(264), 1 << 30, None, None, C.byref(ctx)) == B.ACC_EINVAL
    assert "aligned" in lib.accordion_last_error(None).decode()
    cfgp, keepp = _cfg(method=B.ACC_POWERSGD, level_crit=2, level_noncrit=1)
    assert lib.accordion_init(C.byref(cfgp), C.c_void_p(256), 1 << 30, None, None, C.byref(ctx)) == B.ACC_EINVAL
    assert lib.accordion_init(C.byref(cfg), C.c_void_p(256), 1 << 30, None, None, None) == B.ACC_EINVAL
    # calls on a NULL context fail cleanly
    assert lib.accordion_compress_step(None, 0, None, 0) == B.ACC_EINVAL
    assert lib.accordion_destroy(None) == B.ACC_EINVAL


def test_binding_fails_loudly_when_library_is_missing(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libaccordion.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.load_library()
