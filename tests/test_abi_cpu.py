"""The C-ABI library loads and exports every symbol include/*.h declares; argument
validation answers before anything touches a GPU.  CPU only (no compute calls)."""
import ctypes as C
import os
import re

import pytest

import paper_2504_08966_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:pact|dbdpc)_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = declared_functions()
    assert {"pact_score", "pact_prune", "dbdpc_cluster", "pact_reincorporate", "pact_merge",
            "pact_reduce", "pact_reduce_varlen", "pact_workspace_bytes", "pact_strerror",
            "pact_attention_handoff", "pact_profile_read", "pact_calibration_copy", "pact_plan_workgroups"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name


def test_workspace_size_is_monotone_and_bounded():
    a = P.pact_workspace_bytes(729, 1, 128, 2, 64)
    b = P.pact_workspace_bytes(7290, 1, 512, 4, 128)
    c = P.pact_workspace_bytes(7290, 8, 512, 4, 128)
    assert 0 < a < b < c and b < 64 << 20
    assert P.pact_workspace_bytes(0, 1, 128, 2, 64) == 0
    assert P.pact_workspace_bytes(1 << 20, 1, 128, 2, 64) == 0
    assert P.pact_workspace_bytes(729, 65, 128, 2, 64) == 0
    assert P.pact_workspace_bytes(729, 1, 128, 65, 64) == 0
    # fp32 clustering keys need room for their three-part bf16 copy, bf16 keys do not
    f32 = P.pact_workspace_bytes(7290, 1, 512, 4, 128, P.PACT_F32)
    bf16 = P.pact_workspace_bytes(7290, 1, 512, 4, 128, P.PACT_BF16)
    assert b == f32 and f32 - bf16 >= 7290 * 3 * 512 * 2 and bf16 < 24 << 20
    assert P.load_library().pact_workspace_bytes(729, 1, 128, 7, 2, 64) == 0        # unknown key type


def test_report_layout_matches_the_header():
    """The binding reads the device-side report as 16 words: their order is the struct's."""
    text = open(os.path.join(ROOT, "include", "pact.h")).read()
    body = text[text.index("typedef struct {\n    int32_t n_kept"):text.index("} pact_report;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+([a-z_]+)(?:\[(\d+)\])?;", body)
    names = [f for f, k in fields if f != "reserved"]
    assert tuple(names) == P.REPORT_FIELDS
    assert sum(int(k) if k else 1 for f, k in fields) == 16


def test_non_contiguous_tensors_are_refused():
    import torch
    from paper_2504_08966_amd import binding
    t = torch.zeros(8, 8)
    assert binding._p(t) is not None and binding._p(None) is None
    with pytest.raises(P.PactError):
        binding._p(t[:, ::2])
    with pytest.raises(P.PactError):
        binding._p(t.t())


def test_strerror_covers_all_codes():
    msgs = [P.pact_strerror(i) for i in range(9)]
    assert msgs[0] == "ok" and len(set(msgs)) == 9
    assert P.pact_strerror(99) == "unknown status"


def test_argument_validation_is_host_side():
    """Bad arguments are rejected before any GPU call: NULL pointers, sizes, parameters,
    alignment, workspace.  Fake non-NULL addresses are never dereferenced on these paths."""
    lib = P.load_library()
    fake = C.c_void_p(0x1000)          # 16-byte and 256-byte aligned, never touched
    odd = C.c_void_p(0x1008)
    ws_bytes = 1 << 30
    NULL, SHAPE, DTYPE, PARAM, WS, ALIGN = 1, 2, 3, 4, 5, 6
    # pact_prune
    assert lib.pact_prune(None, 10, 0.5, fake, fake, fake, None, 0, None) == NULL
    assert lib.pact_prune(fake, 0, 0.5, fake, fake, fake, None, 0, None) == SHAPE
    assert lib.pact_prune(fake, 10, 1.5, fake, fake, fake, None, 0, None) == PARAM
    assert lib.pact_prune(fake, 10, float("nan"), fake, fake, fake, None, 0, None) == PARAM
    # pact_score
    sc = lambda **k: lib.pact_score(k.get("hidden", fake), k.get("h_dt", 0), k.get("n", 16), k.get("h", 64),
                                    fake, k.get("k_dt", 0), k.get("n_kv", 2), k.get("d_h", 8), fake, 0,
                                    k.get("q_rows", 16), k.get("n_q", 2), 0, k.get("scores", fake),
                                    k.get("ws", fake), k.get("ws_bytes", ws_bytes), None)
    assert sc(hidden=None) == NULL and sc(scores=None) == NULL
    assert sc(n=0) == SHAPE and sc(n_q=3) == SHAPE and sc(q_rows=5) == SHAPE and sc(n=1 << 20) == SHAPE
    assert sc(h_dt=7) == DTYPE
    assert sc(h=3) == ALIGN and sc(hidden=odd) == ALIGN and sc(d_h=2) == ALIGN
    assert sc(ws=None) == WS and sc(ws_bytes=16) == WS and sc(ws=C.c_void_p(0x1010)) == WS
    # dbdpc_cluster
    db = lambda **k: lib.dbdpc_cluster(k.get("keys", fake), k.get("dt", 1), k.get("n", 16), k.get("dk", 64),
                                       k.get("idx", None), k.get("n_idx", None), k.get("d_c", 0.1),
                                       k.get("d_n", 2.0), k.get("T", 10), fake, fake, fake, None, None,
                                       fake, k.get("ws_bytes", ws_bytes), None)
    assert db(keys=None) == NULL and db(idx=fake) == NULL
    assert db(d_c=-0.1) == PARAM and db(d_n=0.0) == PARAM and db(T=-1) == PARAM
    assert db(d_c=float("inf")) == PARAM
    assert db(dk=4) == ALIGN and db(dt=5) == DTYPE and db(n=-3) == SHAPE and db(ws_bytes=1000) == WS
    # a sample's keys are addressed with 32-bit byte offsets (fp32 keys: 6 bytes per value)
    assert db(n=32768, dk=65536, dt=1) == SHAPE and db(n=32768, dk=24576, dt=0) == SHAPE
    assert db(n=32768, dk=16384, dt=0, ws_bytes=1000) == WS          # within the limit: the next check answers
    # pact_reincorporate / pact_merge
    assert lib.pact_reincorporate(fake, 1, 16, 64, None, fake, 0.1, 1.5, fake, fake, fake, ws_bytes, None) == NULL
    assert lib.pact_reincorporate(fake, 1, 16, 64, fake, fake, 0.1, -1.0, fake, fake, fake, ws_bytes, None) == PARAM
    assert lib.pact_merge(fake, 1, 16, 64, fake, None, fake, 1, fake, 0, fake, fake, ws_bytes, None) == NULL
    assert lib.pact_merge(fake, 1, 16, 64, fake, None, fake, 0, fake, 9, fake, fake, ws_bytes, None) == DTYPE
    assert lib.pact_merge(fake, 1, 16, 60, fake, None, fake, 0, fake, 0, fake, fake, ws_bytes, None) == ALIGN
    # pact_reduce / pact_reduce_varlen
    prm = P.PactParams(0.45, 0.02).c()
    bad_prm = P.PactParams(0.45, 0.02, d_n=-1.0).c()
    rd = lambda p, **k: lib.pact_reduce(fake, 1, k.get("n", 16), 64, fake, k.get("keys", fake), 1, 2, 8, fake,
                                        1, k.get("q_rows", 16), 2, p, fake, fake, fake, fake, fake,
                                        k.get("merged", fake), 0, fake, fake, fake, k.get("ws_bytes", ws_bytes), None)
    assert rd(None) == NULL and rd(C.byref(prm), keys=None) == NULL and rd(C.byref(prm), merged=None) == NULL
    assert rd(C.byref(prm), n=0) == SHAPE and rd(C.byref(prm), q_rows=3) == SHAPE
    assert rd(C.byref(prm), ws_bytes=64) == WS
    # the entry point that brings its own scratch: the same checks, and a size limit instead of a workspace check
    st = lambda p, **k: lib.pact_reduce_static(fake, 1, k.get("n", 16), k.get("h", 64), fake, k.get("keys", fake),
                                               k.get("k_dt", 1), k.get("n_kv", 2), k.get("d_h", 8), fake, 1,
                                               k.get("n", 16), k.get("n_q", 2), p, fake, fake, fake, fake, fake, fake, 0,
                                               fake, fake, None)
    assert st(None) == NULL and st(C.byref(prm), keys=None) == NULL and st(C.byref(bad_prm)) == PARAM
    assert st(C.byref(prm), n=0) == SHAPE
    assert st(C.byref(prm), n=16384, h=3584, k_dt=0, n_kv=4, d_h=128, n_q=4) == WS  # 136 MiB of scratch: refused
    assert P.pact_workspace_bytes(8748, 1, 512, 28, 128, P.PACT_BF16) <= 48 << 20
    bad = P.PactParams(0.45, 0.02, d_n=-1.0).c()
    assert rd(C.byref(bad)) == PARAM
    cu_bad = (C.c_int32 * 3)(0, 8, 8)          # empty second sample
    cu_ok = (C.c_int32 * 3)(0, 8, 16)
    pa = (type(prm) * 2)(prm, prm)
    vl = lambda cu, batch=2, wsb=ws_bytes: lib.pact_reduce_varlen(
        fake, 1, 64, fake, fake, 1, 2, 8, fake, 1, 16, 2, cu, batch, pa, fake, fake, fake, fake, fake, fake,
        0, fake, fake, fake, wsb, None)
    assert vl(cu_bad) == SHAPE and vl(cu_ok, batch=0) == SHAPE and vl(cu_ok, wsb=10) == WS
    assert vl(None) == NULL


def test_valid_call_without_gpu_reports_no_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("this check is for boxes without a GPU")
    lib = P.load_library()
    fake = C.c_void_p(0x1000)
    assert lib.pact_prune(fake, 10, 0.5, fake, fake, fake, None, 0, None) == 8


def test_workgroup_plan_of_a_batch():
    """Host logic behind batched calls: the 256 workgroup slots are dealt to the samples by their tiles."""
    import numpy as np
    import paper_2504_08966_amd as P
    rng = np.random.default_rng(5)
    cases = [[105] * 8, [6, 6, 15, 15, 15, 3, 21, 21, 78, 6, 15, 3, 15, 3, 21, 21], [1] * 64, [2080, 1], [3, 3],
             [300] * 64, [int(x) for x in rng.integers(1, 500, 37)]]
    for tiles in cases:
        wg_map, wg_count = P.pact_plan_workgroups(tiles)
        B = len(tiles)
        assert len(wg_map) == 256 and len(wg_count) == B
        assert all(1 <= c <= t for c, t in zip(wg_count, tiles)) and sum(wg_count) <= 256
        seen = {}
        for slot, e in enumerate(wg_map):
            if e == 0xFFFF:
                continue
            b, rank = e >> 8, e & 255
            assert b < B and rank < wg_count[b] and (b, rank) not in seen
            seen[(b, rank)] = slot
        assert len(seen) == sum(wg_count)                          # every workgroup of every sample has a slot
        # the most loaded workgroup has as few tiles as the slots allow
        turns = max(-(-t // c) for t, c in zip(tiles, wg_count))
        if turns > 1:
            assert sum(-(-t // (turns - 1)) for t in tiles) > 256
        # all slots are used unless every sample already has a workgroup per tile
        assert sum(wg_count) == min(256, sum(tiles))
    # equal samples, a multiple of 8 of them: each sample's workgroups all on one XCD (slot mod 8)
    wg_map, wg_count = P.pact_plan_workgroups([105] * 8)
    assert wg_count == [32] * 8
    for b in range(8):
        assert len({slot % 8 for slot, e in enumerate(wg_map) if e != 0xFFFF and e >> 8 == b}) == 1
    with pytest.raises(P.PactError):
        P.pact_plan_workgroups([0, 5])
    with pytest.raises(P.PactError):
        P.pact_plan_workgroups([5] * 65)
