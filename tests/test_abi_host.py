"""Host-only checks of the C ABI: the library loads, exports what the header declares,
and every argument error is reported before anything could reach a device."""
import os
import re

import numpy as np

import pytest

from paper_2306_08162_amd import binding as ql

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # non-NULL, 16-byte aligned; never dereferenced because validation fails first
ODD = 0x10008           # 8-byte aligned only


def test_library_exports_every_declared_symbol():
    lib = ql.load()
    for fname, exports in (("qlora.h", ql.EXPORTS), ("qlora_bench.h", ql.BENCH_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared = sorted(set(re.findall(r"\b(qlora_[a-z_]+)\s*\(", header)))
        assert declared == sorted(exports), fname
        for name in declared:
            assert hasattr(lib, name), name


def test_status_strings():
    assert ql.status_string(0) == "ok"
    seen = {ql.status_string(i) for i in range(10)}
    assert len(seen) == 10
    assert ql.status_string(99) == "unknown status"


def test_packed_words():
    assert ql.qlora_packed_words(4096, 4096, 4) == 4096 * 512
    assert ql.qlora_packed_words(4096, 11008, 3) == 4096 * 1032
    assert ql.qlora_packed_words(11008, 4096, 2) == 11008 * 256
    assert ql.qlora_packed_words(8, 32, 8) == 8 * 8
    assert ql.qlora_packed_words(8, 32, 5) == 0
    assert ql.qlora_packed_words(8, 48, 4) == 0
    assert ql.qlora_packed_words(7, 32, 4) == 0


def test_workspace_bytes():
    w = ql.qlora_workspace_bytes(2048, 4096, 4096, 4, 128, 8)
    assert w > 0 and w % 256 == 0
    assert ql.qlora_workspace_bytes(2048, 4096, 4096, 4, 128, 0) > 0
    assert ql.qlora_workspace_bytes(0, 4096, 4096, 4, 128, 8) == 0
    assert ql.qlora_workspace_bytes(16, 4096, 4096, 4, 100, 8) == 0
    assert ql.qlora_workspace_bytes(16, 4096, 4096, 4, 128, 12) == 0
    # token counts whose output makes few tiles: room for the fp32 planes of a GEMM split along its contraction
    # (256 x 4096 output = 64 tiles of 128 x 128 -> 4 planes; 512 rows -> 2 planes; 1024 rows: no split)
    assert ql.qlora_workspace_bytes(256, 4096, 4096, 4, 128, 0) >= 4 * 256 * 4096 * 4
    assert ql.qlora_workspace_bytes(512, 4096, 4096, 4, 128, 0) >= 2 * 512 * 4096 * 4
    assert ql.qlora_workspace_bytes(1024, 4096, 4096, 4, 128, 0) < 1024 * 4096 * 4


def _fwd(**kw):
    a = dict(x=FAKE, packed=FAKE, scales=FAKE, zeros=FAKE, A=FAKE, B=FAKE, y=FAKE, t_save=None, M=16, N=64, K=128,
             bits=4, group_size=64, rank=8, alpha=16.0, dtype=0, workspace=FAKE, workspace_bytes=0)
    a.update(kw)
    return ql.qlora_linear_fwd(a["x"], a["packed"], a["scales"], a["zeros"], a["A"], a["B"], a["y"], a["t_save"],
                               a["M"], a["N"], a["K"], a["bits"], a["group_size"], a["rank"], a["alpha"], a["dtype"],
                               a["workspace"], a["workspace_bytes"], stream=0, check=False)


def _bwd(**kw):
    a = dict(dy=FAKE, x=FAKE, packed=FAKE, scales=FAKE, zeros=FAKE, A=FAKE, B=FAKE, t_saved=None, dx=FAKE, dA=FAKE,
             dB=FAKE, M=16, N=64, K=128, bits=4, group_size=64, rank=8, alpha=16.0, dtype=0, workspace=FAKE,
             workspace_bytes=0)
    a.update(kw)
    return ql.qlora_linear_bwd(a["dy"], a["x"], a["packed"], a["scales"], a["zeros"], a["A"], a["B"], a["t_saved"],
                               a["dx"], a["dA"], a["dB"], a["M"], a["N"], a["K"], a["bits"], a["group_size"],
                               a["rank"], a["alpha"], a["dtype"], a["workspace"], a["workspace_bytes"], stream=0,
                               check=False)


E = {n: i for i, n in enumerate(ql.STATUS_NAMES)}


@pytest.mark.parametrize("call", [_fwd, _bwd], ids=["fwd", "bwd"])
def test_linear_argument_errors(call):
    assert call(bits=5) == E["QLORA_E_BITS"]
    assert call(bits=1) == E["QLORA_E_BITS"]
    assert call(M=0) == E["QLORA_E_SHAPE"]
    assert call(K=48) == E["QLORA_E_SHAPE"]
    assert call(N=60) == E["QLORA_E_SHAPE"]
    assert call(M=1 << 20, K=4096) == E["QLORA_E_SHAPE"]
    assert call(group_size=48) == E["QLORA_E_GROUP"]
    assert call(group_size=96) == E["QLORA_E_GROUP"]      # 128 % 96 != 0
    assert call(group_size=0) == E["QLORA_E_GROUP"]
    assert call(rank=4) == E["QLORA_E_RANK"]
    assert call(rank=72) == E["QLORA_E_RANK"]
    assert call(rank=-8) == E["QLORA_E_RANK"]
    assert call(dtype=2) == E["QLORA_E_DTYPE"]
    assert call(packed=None) == E["QLORA_E_NULL"]
    assert call(scales=None) == E["QLORA_E_NULL"]
    assert call(zeros=None) == E["QLORA_E_NULL"]
    assert call(A=None) == E["QLORA_E_NULL"]
    assert call(B=None) == E["QLORA_E_NULL"]
    assert call(packed=ODD) == E["QLORA_E_ALIGN"]
    assert call(A=ODD) == E["QLORA_E_ALIGN"]
    assert call(workspace=ODD) == E["QLORA_E_ALIGN"]
    # everything valid except the workspace: still refused before any launch
    assert call(workspace_bytes=0) == E["QLORA_E_WORKSPACE"]
    assert call(workspace=None, workspace_bytes=1 << 30) == E["QLORA_E_WORKSPACE"]
    need = ql.qlora_workspace_bytes(16, 64, 128, 4, 64, 8)
    assert call(workspace_bytes=need - 1) == E["QLORA_E_WORKSPACE"]
    # rank 0: adapters may be NULL, the check then moves on to the workspace
    assert call(rank=0, A=None, B=None) == E["QLORA_E_WORKSPACE"]


def test_fwd_bwd_specific_null_checks():
    assert _fwd(x=None) == E["QLORA_E_NULL"]
    assert _fwd(y=None) == E["QLORA_E_NULL"]
    assert _bwd(dy=None) == E["QLORA_E_NULL"]
    assert _bwd(dx=None) == E["QLORA_E_NULL"]
    assert _bwd(dA=None) == E["QLORA_E_NULL"]
    assert _bwd(dB=None) == E["QLORA_E_NULL"]
    assert _bwd(x=None) == E["QLORA_E_NULL"]
    assert _bwd(rank=0, x=None, A=None, B=None, dA=None, dB=None) == E["QLORA_E_WORKSPACE"]
    assert _bwd(dA=ODD) == E["QLORA_E_ALIGN"]


def _sib(which, count=2, N=(64, 40), M=4, K=128, bits=4, G=64, rank=8, dtype=0, ws=FAKE, ws_bytes=1 << 30, **over):
    """A sibling call with fake pointers; `over` replaces one argument (a list, a pointer or None)."""
    a = dict(x=FAKE, packed=[FAKE] * count, scales=[FAKE] * count, zeros=[FAKE] * count, A=[FAKE] * count,
             B=[FAKE] * count, y=[FAKE] * count, t=None, dy=[FAKE] * count, dx=FAKE, dA=[FAKE] * count,
             dB=[FAKE] * count)
    a.update(over)
    N = list(N)[:count] if len(N) >= count else list(N) + [64] * (count - len(N))
    if which == "fwd":
        return ql.qlora_linear_fwd_siblings(a["x"], a["packed"], a["scales"], a["zeros"], a["A"], a["B"], a["y"],
                                            a["t"], N, M, K, bits, G, rank, 16.0, dtype, ws, ws_bytes, stream=0,
                                            check=False)
    return ql.qlora_linear_bwd_siblings(a["dy"], a["x"], a["packed"], a["scales"], a["zeros"], a["A"], a["B"], a["t"],
                                        a["dx"], a["dA"], a["dB"], N, M, K, bits, G, rank, 16.0, dtype, ws, ws_bytes,
                                        stream=0, check=False)


@pytest.mark.parametrize("which", ["fwd", "bwd"])
def test_sibling_argument_errors(which):
    assert _sib(which, M=17) == E["QLORA_E_SHAPE"]                 # only the weight-streaming regime
    assert _sib(which, count=5, N=(64,) * 5) == E["QLORA_E_SHAPE"]
    assert _sib(which, N=(64, 44)) == E["QLORA_E_SHAPE"]           # N % 8
    assert _sib(which, bits=5) == E["QLORA_E_BITS"]
    assert _sib(which, G=48) == E["QLORA_E_GROUP"]
    assert _sib(which, rank=12) == E["QLORA_E_RANK"]
    assert _sib(which, dtype=2) == E["QLORA_E_DTYPE"]
    assert _sib(which, packed=[FAKE, None]) == E["QLORA_E_NULL"]
    assert _sib(which, B=[None, FAKE]) == E["QLORA_E_NULL"]
    assert _sib(which, scales=None) == E["QLORA_E_NULL"]
    assert _sib(which, zeros=[FAKE, ODD]) == E["QLORA_E_ALIGN"]
    assert _sib(which, x=None) == E["QLORA_E_NULL"]
    need = ql.qlora_siblings_workspace_bytes([64, 40], 4, 128, 4, 64, 8)
    assert need > 0
    assert _sib(which, ws_bytes=need - 1) == E["QLORA_E_WORKSPACE"]
    assert _sib(which, ws=None) == E["QLORA_E_WORKSPACE"]
    assert _sib(which, rank=0, A=None, B=None, dA=None, dB=None, ws_bytes=0) == E["QLORA_E_WORKSPACE"]
    if which == "bwd":
        assert _sib(which, dA=[FAKE, None]) == E["QLORA_E_NULL"]
        assert _sib(which, dx=None) == E["QLORA_E_NULL"]
        assert _sib(which, dy=[None, FAKE]) == E["QLORA_E_NULL"]
    else:
        assert _sib(which, y=[FAKE, None]) == E["QLORA_E_NULL"]


def test_bwd_accumulate_argument_errors():
    args = [FAKE] * 11
    def call(beta=1.0, M=16, N=64, K=128, bits=4, G=64, rank=8, dtype=0, dA=FAKE, wsb=1 << 30):
        a = list(args)
        a[9] = dA
        return ql.qlora_linear_bwd_accumulate(*a, beta, M, N, K, bits, G, rank, 16.0, dtype, FAKE, wsb, stream=0,
                                              check=False)
    assert call(bits=5) == E["QLORA_E_BITS"]
    assert call(rank=12) == E["QLORA_E_RANK"]
    assert call(dA=None) == E["QLORA_E_NULL"]
    assert call(wsb=0) == E["QLORA_E_WORKSPACE"]


def test_dropout_argument_errors():
    def fwd(mask=FAKE, **kw):
        d = dict(M=16, N=64, K=128, bits=4, G=64, rank=8, dtype=0, wsb=1 << 30)
        d.update(kw)
        return ql.qlora_linear_fwd_dropout(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, mask, 1.0 / 0.95, FAKE, FAKE, d["M"],
                                           d["N"], d["K"], d["bits"], d["G"], d["rank"], 16.0, d["dtype"], FAKE,
                                           d["wsb"], stream=0, check=False)

    def bwd(mask=FAKE, **kw):
        d = dict(M=16, N=64, K=128, bits=4, G=64, rank=8, dtype=0, wsb=1 << 30)
        d.update(kw)
        return ql.qlora_linear_bwd_dropout(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, mask, 1.0 / 0.95, FAKE, FAKE, FAKE,
                                           FAKE, 0.0, d["M"], d["N"], d["K"], d["bits"], d["G"], d["rank"], 16.0,
                                           d["dtype"], FAKE, d["wsb"], stream=0, check=False)

    for call in (fwd, bwd):
        assert call(bits=7) == E["QLORA_E_BITS"]
        assert call(K=100) == E["QLORA_E_SHAPE"]
        assert call(mask=ODD) == E["QLORA_E_ALIGN"]
        assert call(wsb=0) == E["QLORA_E_WORKSPACE"]
        assert call(mask=None, wsb=0) == E["QLORA_E_WORKSPACE"]       # no mask is allowed: plain layer


def test_sibling_workspace_bytes():
    assert ql.qlora_siblings_workspace_bytes([64, 40], 17, 128, 4, 64, 8) == 0
    assert ql.qlora_siblings_workspace_bytes([64, 44], 4, 128, 4, 64, 8) == 0
    one = ql.qlora_siblings_workspace_bytes([4096], 16, 4096, 4, 128, 8)
    three = ql.qlora_siblings_workspace_bytes([4096] * 3, 16, 4096, 4, 128, 8)
    # both hold the dX row slices of one launch of about 256 workgroups, so they are of one size class
    assert one >= 16 * 4096 * 4 and three >= 16 * 4096 * 4 and three < 4 * one


def test_lrec_loss_argument_errors():
    def call(M=4, V=64, dtype=0, zs=FAKE, zt=FAKE, lab=FAKE, kl=FAKE, ce=FAKE, mean=FAKE, grad=FAKE, ws=FAKE, wsb=1 << 20):
        return ql.qlora_lrec_loss(zs, zt, lab, 1.0, 120.0, kl, ce, mean, grad, M, V, dtype, ws, wsb, stream=0, check=False)
    assert call(M=0) == E["QLORA_E_SHAPE"]
    assert call(V=60) == E["QLORA_E_SHAPE"]             # V % 8
    assert call(V=0) == E["QLORA_E_SHAPE"]
    assert call(dtype=3) == E["QLORA_E_DTYPE"]
    assert call(zs=None) == E["QLORA_E_NULL"]
    assert call(zt=None) == E["QLORA_E_NULL"]
    assert call(lab=None) == E["QLORA_E_NULL"]
    assert call(mean=None) == E["QLORA_E_NULL"]
    assert call(zs=ODD) == E["QLORA_E_ALIGN"]
    assert call(grad=ODD) == E["QLORA_E_ALIGN"]
    assert call(kl=0x10002) == E["QLORA_E_ALIGN"]
    assert call(ws=None) == E["QLORA_E_WORKSPACE"]
    assert call(wsb=ql.qlora_lrec_workspace_bytes(4) - 1) == E["QLORA_E_WORKSPACE"]
    assert ql.qlora_lrec_workspace_bytes(0) == 0 and ql.qlora_lrec_workspace_bytes(2048) >= 2048 * 4


def test_pack_unpack_argument_errors():
    for fn in (ql.qlora_pack, ql.qlora_unpack):
        assert fn(FAKE, FAKE, 8, 64, 5, stream=0, check=False) == E["QLORA_E_BITS"]
        assert fn(FAKE, FAKE, 8, 40, 4, stream=0, check=False) == E["QLORA_E_SHAPE"]
        assert fn(FAKE, FAKE, 0, 64, 4, stream=0, check=False) == E["QLORA_E_SHAPE"]
        assert fn(None, FAKE, 8, 64, 4, stream=0, check=False) == E["QLORA_E_NULL"]
        assert fn(FAKE, None, 8, 64, 4, stream=0, check=False) == E["QLORA_E_NULL"]
        assert fn(ODD, FAKE, 8, 64, 4, stream=0, check=False) == E["QLORA_E_ALIGN"]


def test_error_raises_with_check():
    with pytest.raises(ql.QLoraError) as ei:
        ql.qlora_pack(FAKE, FAKE, 8, 64, 7, stream=0)
    assert ei.value.status == E["QLORA_E_BITS"]


def test_actorder_perm_host_function_and_its_errors():
    """qlora_actorder_perm is pure host work: checked here against numpy's stable sort, plus its error paths."""
    from paper_2306_08162_amd import workloads as wl
    K, G = 384, 32
    g_idx = wl.actorder_g_idx(17, K, G)
    perm = np.empty(K, dtype=np.int32)
    inv = np.empty(K, dtype=np.int32)
    assert ql.qlora_actorder_perm(g_idx, perm, inv, K, G, check=False) == 0
    ref = np.argsort(g_idx, kind="stable")
    assert np.array_equal(perm, ref) and np.array_equal(inv[ref], np.arange(K))
    assert ql.qlora_actorder_perm(g_idx, perm, None, K, G, check=False) == 0          # inverse is optional
    bad = g_idx.copy()
    bad[5] = K // G
    assert ql.qlora_actorder_perm(bad, perm, inv, K, G, check=False) == ql.STATUS_NAMES.index("QLORA_E_GIDX")
    bad = g_idx.copy()
    bad[5] = (bad[5] + 1) % (K // G)                                                  # one group too full
    assert ql.qlora_actorder_perm(bad, perm, inv, K, G, check=False) == ql.STATUS_NAMES.index("QLORA_E_GIDX")
    assert ql.qlora_actorder_perm(None, perm, inv, K, G, check=False) == ql.STATUS_NAMES.index("QLORA_E_NULL")
    assert ql.qlora_actorder_perm(g_idx, perm, inv, K, 48, check=False) == ql.STATUS_NAMES.index("QLORA_E_GROUP")
    assert ql.qlora_actorder_perm(g_idx, perm, inv, 40, 32, check=False) == ql.STATUS_NAMES.index("QLORA_E_SHAPE")
    assert ql.qlora_pack_permuted(None, None, None, 8, 64, 4, stream=0, check=False) == ql.STATUS_NAMES.index("QLORA_E_NULL")
    assert ql.qlora_pack_permuted(None, None, None, 8, 64, 5, stream=0, check=False) == ql.STATUS_NAMES.index("QLORA_E_BITS")
    assert ql.qlora_gather_columns(None, None, None, 4, 64, stream=0, check=False) == ql.STATUS_NAMES.index("QLORA_E_NULL")
    assert ql.qlora_gather_columns(None, None, None, 0, 64, stream=0, check=False) == ql.STATUS_NAMES.index("QLORA_E_SHAPE")
    assert ql.qlora_gather_columns(None, None, None, 4, 40, stream=0, check=False) == ql.STATUS_NAMES.index("QLORA_E_SHAPE")


def test_packed_zero_words_and_errors():
    assert ql.qlora_packed_zero_words(4096, 32, 4) == 4096 * 4
    assert ql.qlora_packed_zero_words(8, 11, 3) == 8 * 2
    assert ql.qlora_packed_zero_words(8, 1, 2) == 8
    assert ql.qlora_packed_zero_words(8, 11, 5) == 0 and ql.qlora_packed_zero_words(0, 11, 4) == 0
    E = ql.STATUS_NAMES.index
    assert ql.qlora_pack_zeros(None, None, 8, 4, 4, stream=0, check=False) == E("QLORA_E_NULL")
    assert ql.qlora_unpack_zeros(None, None, 8, 4, 6, stream=0, check=False) == E("QLORA_E_BITS")
    assert ql.qlora_unpack_zeros(None, None, 8, 0, 4, stream=0, check=False) == E("QLORA_E_SHAPE")


def test_stacked_backward_rejects_bad_frozen_rank():
    E = ql.STATUS_NAMES.index
    args = lambda frozen, rank: ql.qlora_linear_bwd_stacked(None, None, None, None, None, None, None, None, None, None, None,
                                                             0.0, frozen, 32, 64, 128, 4, 64, rank, 16.0, ql.QLORA_F16, None, 0,
                                                             stream=0, check=False)
    assert args(4, 16) == E("QLORA_E_RANK")          # not a multiple of 8
    assert args(16, 16) == E("QLORA_E_RANK")         # nothing left to train
    assert args(-8, 16) == E("QLORA_E_RANK")
    assert args(8, 16) == E("QLORA_E_NULL")          # accepted, then the NULL buffers are caught


def test_bench_refuses_more_than_one_gpu():
    """The layer has no multi-GPU path: bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
