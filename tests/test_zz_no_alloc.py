"""graphkv_compress_static (the entry point for callers that cannot allocate) against
graphkv_compress, through the C ABI: same bytes, on two calls in a row that share the built-in
scratch buffer, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2509_00388_amd import binding as gk
from paper_2509_00388_amd import synth
from tests import util

pytestmark = pytest.mark.gpu


def outputs(p):
    shape = (p.n_kv_heads, p.budget, p.head_dim)
    return (torch.zeros(shape, dtype=p.torch_dtype, device="cuda"), torch.zeros(shape, dtype=p.torch_dtype, device="cuda"),
            torch.zeros((p.n_kv_heads, p.budget), dtype=torch.int32, device="cuda"),
            torch.zeros((p.n_kv_heads, p.n_prefix), dtype=torch.float32, device="cuda"))


def test_static_scratch_entry_equals_workspace_entry():
    c2 = synth.CONFIGS["c2"]
    cases = [(synth.scaled(c2, n_tokens=9100, n_sources=40, n_neighbors=12, budget=700, n_kv_heads=2, n_q_heads=8),
              dict(rounds=3)),                                                    # filter route, lists kept
             (synth.scaled(c2, n_tokens=1500, budget=200, n_sources=16, n_neighbors=8, n_kv_heads=2, n_q_heads=8),
              dict(rounds=2)),                                                    # smaller: dense route
             (synth.scaled(c2, n_tokens=700, budget=90, n_sources=5, n_neighbors=3, n_kv_heads=1, n_q_heads=4),
              dict(rounds=1, scorer=gk.SCORER_KNORM))]
    prepared = []
    for cfg, kw in cases:
        host, dev = util.device_layer(cfg, 1)
        p = util.params_from_cfg(cfg, **kw)
        assert 0 < gk.graphkv_workspace_bytes(p) <= gk.STATIC_SCRATCH_BYTES
        want = outputs(p)
        gk.graphkv_compress(p, *dev, want[0], want[1], want[2], scores_out=want[3])
        prepared.append((p, dev, want, outputs(p)))
    torch.cuda.synchronize()
    # the calls under test, back to back on the one built-in buffer, no allocation in between
    for p, dev, want, got in prepared:
        print(f"static-scratch call N={p.n_tokens}", flush=True)
        gk.graphkv_compress_static(p, *dev, got[0], got[1], got[2], scores_out=got[3])
    torch.cuda.synchronize()
    for p, dev, want, got in prepared:
        assert torch.equal(got[2], want[2]), f"N={p.n_tokens}: indices"
        assert torch.equal(got[0].view(torch.int16), want[0].view(torch.int16)), "gathered keys"
        assert torch.equal(got[1].view(torch.int16), want[1].view(torch.int16)), "gathered values"
        assert np.array_equal(got[3].cpu().numpy(), want[3].cpu().numpy(), equal_nan=True), "refined scores"
        assert int(got[2].max()) == p.n_tokens - 1


def test_static_scratch_entry_rejects_what_does_not_fit():
    cfg = synth.CONFIGS["c5"]
    p = util.params_from_cfg(cfg)
    assert gk.graphkv_workspace_bytes(p) > gk.STATIC_SCRATCH_BYTES
    cfg_s = synth.scaled(synth.CONFIGS["c2"], n_tokens=700, budget=90, n_kv_heads=1, n_q_heads=4)
    host, dev = util.device_layer(cfg_s, 0)
    o = outputs(util.params_from_cfg(cfg_s))
    with pytest.raises(gk.GraphKVError, match="-4"):
        # (buffers of the small problem, params of the large one: the size check comes first)
        lib = gk.load_library()
        import ctypes
        cp = p.c()
        gk._check(lib.graphkv_compress_static(ctypes.byref(cp), dev[0].data_ptr(), dev[1].data_ptr(), dev[2].data_ptr(),
                                              o[0].data_ptr(), o[1].data_ptr(), o[2].data_ptr(), None, None))
