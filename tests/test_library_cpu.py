"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2509_00388_amd import binding as gk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gk.LIB_PATH):
        from paper_2509_00388_amd import build
        build.build()
    return gk.load_library()


def good_params(**kw):
    p = gk.Params(n_kv_heads=8, n_q_heads=32, head_dim=128, n_tokens=4096, window=32, pool_kernel=7,
                  budget=512, n_sources=32, n_neighbors=8, rounds=1, dtype=gk.BF16)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "graphkv.h")).read()
    declared = set(re.findall(r"\b(graphkv_[a-z_]+)\s*\(", header))
    assert declared == set(gk.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_params_struct_layout_matches_header():
    header = open(os.path.join(ROOT, "include", "graphkv.h")).read()
    body = header.split("typedef struct graphkv_params {")[1].split("} graphkv_params;")[0]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|float)\s+([a-z_]+);", body)
    want = [(("float" if f[1] is ctypes.c_float else "int32_t"), f[0]) for f in gk._CParams._fields_]
    assert fields == want
    assert ctypes.sizeof(gk._CParams) == 4 * len(want)


def test_workspace_size_and_mfma_choice(lib):
    p = good_params()
    assert gk.graphkv_workspace_bytes(p) > 0
    assert gk.graphkv_workspace_bytes(good_params(head_dim=12)) == 0
    assert gk.graphkv_uses_mfma(p)
    assert not gk.graphkv_uses_mfma(good_params(impl=gk.IMPL_GENERIC))
    assert not gk.graphkv_uses_mfma(good_params(dtype=gk.FP32))
    assert not gk.graphkv_uses_mfma(good_params(head_dim=64))
    assert gk.graphkv_uses_mfma(good_params(window=64))        # 4 * 64 = 256 rows: two parts
    assert not gk.graphkv_uses_mfma(good_params(window=96))    # 384 rows
    # the generic path stores the logits, the MFMA path does not
    assert gk.graphkv_workspace_bytes(good_params(impl=gk.IMPL_GENERIC)) > gk.graphkv_workspace_bytes(p)


def test_batched_workspace_stays_bounded(lib):
    """The edge block of the overflow path is never carved in full: the long-context workload
    (32 layers x 8 heads, N = 131072, S = m = 128) needs less than 2 GiB of scratch, the 32K one
    less than 1 GiB."""
    c5 = good_params(n_tokens=131072, window=64, budget=4096, n_sources=128, n_neighbors=128, rounds=3)
    c3 = good_params(n_tokens=32768, window=32, budget=2048, n_sources=64, n_neighbors=32, rounds=2)
    assert 0 < gk.graphkv_workspace_bytes_batched(c5, 32) < 2 << 30
    assert 0 < gk.graphkv_workspace_bytes_batched(c3, 32) < 1 << 30
    assert gk.graphkv_workspace_bytes(c3) <= gk.STATIC_SCRATCH_BYTES    # a 32K layer fits the built-in buffer
    # a batch whose scratch would pass the bound is cut into launch groups: 32 layers then ask for
    # what 16 ask for
    wide = good_params(n_tokens=32768, window=32, budget=2048, n_sources=224, n_neighbors=400, rounds=2)
    assert gk.graphkv_workspace_bytes_batched(wide, 32) == gk.graphkv_workspace_bytes_batched(wide, 16) < 2000 << 20
    assert gk.graphkv_workspace_bytes_batched(wide, 8) < gk.graphkv_workspace_bytes_batched(wide, 16)


BAD = [dict(n_kv_heads=0), dict(n_q_heads=12), dict(head_dim=100), dict(head_dim=1024),
       dict(window=0), dict(window=4096), dict(pool_kernel=4), dict(pool_kernel=0), dict(pool_mode=2),
       dict(budget=32), dict(budget=4097), dict(n_sources=0), dict(n_sources=4065),
       dict(n_neighbors=0), dict(n_neighbors=4064), dict(rounds=-1), dict(decay=1.5),
       dict(decay=-0.1), dict(decay=float("nan")), dict(reselect=2), dict(dtype=3),
       dict(softmax_scale=-1.0), dict(signal=3), dict(impl=2)]


@pytest.mark.parametrize("kw", BAD)
def test_invalid_params_are_rejected_on_the_host(lib, kw):
    """Fake but aligned pointers: validation must fail before any of them is used."""
    cp = good_params(**kw).c()
    fake = ctypes.c_void_p(0x10000)
    rc = lib.graphkv_compress(ctypes.byref(cp), fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None)
    assert rc == -1, kw
    assert "invalid" in gk.graphkv_strerror(rc)


def test_null_misaligned_and_small_workspace(lib):
    cp = good_params().c()
    fake = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10004)
    need = lib.graphkv_workspace_bytes(ctypes.byref(cp))
    assert lib.graphkv_compress(ctypes.byref(cp), None, fake, fake, fake, fake, fake, None, fake, need, None) == -1
    assert lib.graphkv_compress(ctypes.byref(cp), odd, fake, fake, fake, fake, fake, None, fake, need, None) == -1
    assert lib.graphkv_compress(ctypes.byref(cp), fake, fake, fake, fake, fake, fake, None, fake, need - 1, None) == -2
    assert lib.graphkv_compress(ctypes.byref(cp), fake, fake, fake, fake, fake, fake, None, None, need, None) == -2
    assert lib.graphkv_score(ctypes.byref(cp), fake, fake, fake, odd, need, None) == -2
    assert lib.graphkv_propagate(ctypes.byref(cp), fake, None, None, None, None, fake, need, None) == -1
    assert lib.graphkv_select(ctypes.byref(cp), None, fake, None, 0, None) == -1
    assert "workspace" in gk.graphkv_strerror(-2)
    assert gk.graphkv_strerror(-3) and gk.graphkv_strerror(-99)


def test_score_call_sizes_its_scratch_for_the_attention_scorer(lib):
    """graphkv_score is the attention scorer whatever the params' scorer field says: a workspace
    sized for key-norm params (no logits, no votes) is turned down, not overrun."""
    fake = ctypes.c_void_p(0x10000)
    for impl in (gk.IMPL_AUTO, gk.IMPL_GENERIC):
        att, kn = good_params(impl=impl), good_params(impl=impl, scorer=gk.SCORER_KNORM)
        need_att, need_kn = gk.graphkv_workspace_bytes(att), gk.graphkv_workspace_bytes(kn)
        assert need_kn <= need_att
        cp = kn.c()
        if need_kn < need_att:
            assert lib.graphkv_score(ctypes.byref(cp), fake, fake, fake, fake, need_kn, None) == -2
    generic = good_params(impl=gk.IMPL_GENERIC)
    assert gk.graphkv_workspace_bytes(good_params(impl=gk.IMPL_GENERIC, scorer=gk.SCORER_KNORM)) < \
        gk.graphkv_workspace_bytes(generic)


def test_static_scratch_entry_checks_on_the_host(lib):
    """graphkv_compress_static: invalid params and problems beyond its built-in buffer are turned
    down before anything touches a GPU."""
    fake = ctypes.c_void_p(0x10000)
    big = good_params(n_tokens=131072, window=64, budget=4096, n_sources=128, n_neighbors=128, rounds=3).c()
    assert lib.graphkv_workspace_bytes(ctypes.byref(big)) > gk.STATIC_SCRATCH_BYTES
    assert lib.graphkv_compress_static(ctypes.byref(big), fake, fake, fake, fake, fake, fake, None, None) == -4
    assert "scratch" in gk.graphkv_strerror(-4)
    bad = good_params(head_dim=100).c()
    assert lib.graphkv_compress_static(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, None, None) == -1
    ok = good_params().c()
    assert lib.graphkv_workspace_bytes(ctypes.byref(ok)) <= gk.STATIC_SCRATCH_BYTES
    assert lib.graphkv_compress_static(ctypes.byref(ok), None, fake, fake, fake, fake, fake, None, None) == -1
    header = open(os.path.join(ROOT, "include", "graphkv.h")).read()
    assert re.search(r"#define GRAPHKV_STATIC_SCRATCH_BYTES \(\(size_t\)64 << 20\)", header)


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(gk, "_lib", None)
    monkeypatch.setattr(gk, "LIB_PATH", "/nonexistent/libgraphkv.so")
    with pytest.raises(gk.GraphKVError):
        gk.load_library()
