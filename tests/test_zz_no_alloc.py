"""pact_reduce_static (the entry point that takes no workspace and allocates nothing) against
pact_reduce, through the C ABI: two calls in a row on the library's one scratch array, the second
on a smaller input, every output compared bit for bit (the kernels are the same)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2504_08966_amd as P
from pact_synth import gen
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

KEYS = ("scores", "kept_idx", "pruned_idx", "center_idx", "cluster_id", "cluster_counts", "merged")


def _both(name, seed, out_dtype=torch.float32, first=False):
    s = gen.make_sample(name, seed)
    cfg = s.config
    d = gu.sample_to_dev(s)
    prm = P.PactParams(s.lam, gu.d_c_of(s), 2.0, 1.5)
    ref = P.pact_reduce(d["hidden"], d["keys"], d["keys"], d["q"], cfg.n_kv, cfg.d_h, cfg.n_kv, prm, out_dtype=out_dtype)
    torch.cuda.synchronize()
    out = P.new_outputs(s.n, cfg.hidden, 1, out_dtype)
    for k in KEYS:
        out[k].view(torch.uint8).fill_(0xEE)                       # poison: whatever is compared was written by the call
    free_before = torch.cuda.mem_get_info()[0]
    P.pact_reduce_static(d["hidden"], d["keys"], d["keys"], d["q"], cfg.n_kv, cfg.d_h, cfg.n_kv, prm, out)
    torch.cuda.synchronize()
    # (the first use of the array on a device is when the runtime loads the code object that holds it)
    assert first or torch.cuda.mem_get_info()[0] == free_before     # the device's free memory did not move
    return s, gu.trim(ref, s.n), gu.trim(out, s.n)


def _same(a, b, what):
    # (the number of centre rounds depends on how the wavefronts of a round interleave; the centres do not)
    strip = lambda r: {k: v for k, v in r.items() if k != "rounds"}
    assert strip(a["rep"]) == strip(b["rep"]), what
    for k in ("scores", "kept_idx", "pruned_idx", "center_idx", "cluster_id", "counts", "merged"):
        assert np.array_equal(a[k], b[k]), f"{what}: {k} differs"


def test_static_scratch_entry_point_equals_pact_reduce():
    s1, ref1, got1 = _both("img_7b", 0, first=True)                 # 20.8 MiB of the 48 MiB array
    _same(ref1, got1, "first call (7290 tokens)")
    assert got1["rep"]["n_centers"] == gu.manifest()[gu.sample_key(s1)]["C"]
    s2, ref2, got2 = _both("tiny_bf16", 2, torch.bfloat16)          # smaller input, the array holds the first call's data
    _same(ref2, got2, "second call (392 tokens)")
    s3, ref3, got3 = _both("img_0p5b", 1)                           # fp32 keys: the three-part copy lives in the array too
    _same(ref3, got3, "third call (729 tokens, fp32 keys)")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    s = gen.make_sample("tiny_f32", 0)
    cfg = s.config
    d = gu.sample_to_dev(s)
    out = P.new_outputs(s.n, cfg.hidden)
    lib = P.load_library()
    prm = P.PactParams(0.5, 0.02).c()
    p = lambda t: C.c_void_p(t.data_ptr())
    # claimed sizes whose workspace would exceed the array: refused on the host, nothing is touched
    assert P.pact_workspace_bytes(16384, 1, 512, 4, 128, P.PACT_F32) > 48 << 20
    rc = lib.pact_reduce_static(p(d["hidden"]), 0, 16384, cfg.hidden, p(d["keys"]), p(d["keys"]), 0, 4, 128, p(d["q"]), 0,
                                16384, 4, C.byref(prm), p(out["scores"]), p(out["kept_idx"]), p(out["pruned_idx"]),
                                p(out["center_idx"]), p(out["cluster_id"]), p(out["merged"]), 0,
                                p(out["cluster_counts"]), p(out["rep"]), None)
    assert rc == 5 and "workspace" in P.pact_strerror(rc)
    assert lib.pact_reduce_static(None, 0, 16, 64, None, None, 0, 2, 8, None, 0, 16, 2, C.byref(prm), None, None, None,
                                  None, None, None, 0, None, None, None) == 1
