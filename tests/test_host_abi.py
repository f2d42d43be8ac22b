"""CPU-only tests of the C ABI: the library loads and exports every symbol the
header declares, the plan builder validates and tiles the layer table, and the
host functions (finalize, rank) agree with the oracle.  No kernel is launched."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from oracle import reference as orc
from paper_2501_07161_amd import binding as qb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000          # stands in for a device address; never dereferenced on the host


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "qv2.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(qv2_[a-z0-9_]+)\s*\(", hdr))
    assert {"qv2_calibrate", "qv2_fakequant_metrics", "qv2_pair_metrics", "qv2_rank"} <= declared
    L = ctypes.CDLL(qb.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(qb.EXPORTS)


def test_struct_layouts_match_header_sizes():
    assert ctypes.sizeof(qb.qv2_tensor) == 48
    assert ctypes.sizeof(qb.qv2_rank_config) == 40
    c = qb.qv2_rank_config_default()
    assert (c.alpha_w, c.alpha_a, c.mse_factor, c.sqnr_cap_db, c.mse_source) == (0.6, 0.4, 5.0, 200.0, 0)


def test_status_strings():
    for st in range(-10, 1):
        assert qb.lib().qv2_status_string(st) and qb.lib().qv2_status_string(st) != b"unknown status"
    assert b"unknown" in qb.lib().qv2_status_string(-99)


def _row(numel, scheme=qb.QV2_ASYM_TENSOR, channels=1, x=FAKE, qrun=None, codes=None, kind=0, layer=0):
    return qb.TensorArg(x=x, numel=numel, scheme=scheme, channels=channels, qrun=qrun, codes=codes,
                        kind=kind, layer=layer)


@pytest.mark.parametrize("row,status", [
    (_row(0), qb.QV2_ERR_SHAPE),
    (_row(-5), qb.QV2_ERR_SHAPE),
    (_row(100, channels=2), qb.QV2_ERR_SHAPE),                       # per-tensor needs channels == 1
    (_row(100, qb.QV2_SYM_CHANNEL, channels=7), qb.QV2_ERR_SHAPE),   # 7 does not divide 100
    (_row(100, qb.QV2_SYM_CHANNEL, channels=0), qb.QV2_ERR_SHAPE),
    (_row(100, scheme=3), qb.QV2_ERR_SCHEME),
    (_row(100, scheme=-1), qb.QV2_ERR_SCHEME),
    (_row(100, x=None), qb.QV2_ERR_NULL),
    (_row(100, x=FAKE + 2), qb.QV2_ERR_ALIGN),
    (_row(100, qrun=FAKE + 1), qb.QV2_ERR_ALIGN),
])
def test_plan_rejects_bad_rows(row, status):
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_plan_create([_row(64), row])
    assert e.value.status == status


def test_plan_rejects_empty_and_null():
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_plan_create([])
    assert e.value.status == qb.QV2_ERR_SHAPE
    h = ctypes.c_void_p()
    assert qb.lib().qv2_plan_create(None, 1, ctypes.byref(h)) == qb.QV2_ERR_NULL
    arr = (qb.qv2_tensor * 1)()
    assert qb.lib().qv2_plan_create(arr, 1, None) == qb.QV2_ERR_NULL
    assert qb.lib().qv2_plan_num_segments(None) == 0
    qb.lib().qv2_plan_destroy(None)


def test_plan_tiling_counts():
    TR, TQ = 32768, 2048                                        # default read / quantize stream tiles
    rows = [
        _row(200_704, qrun=FAKE, codes=FAKE),                   # 7 read tiles (6 full + 4096), 98 quantize tiles
        _row(9408, codes=FAKE),                                 # 1 read tile, 5 quantize tiles
        _row(32 * 9, qb.QV2_SYM_CHANNEL, 32),                   # 16 lanes per row, 16 rows per 256-thread tile -> 2 tiles
        _row(4096 * 40000, qb.QV2_SYM_CHANNEL, 4096, codes=FAKE),   # rows longer than a tile: 2 / 20 tiles each
        _row(2048 * 512, qb.QV2_SYM_CHANNEL, 2048),             # aligned rows of 512: 16 lanes per row, 16 rows per 256-thread tile -> 128 tiles
        _row(3000 * 3, qb.QV2_SYM_CHANNEL, 3000),               # 4 lanes per row: 64 rows per tile -> 47 tiles
    ]
    p = qb.qv2_plan_create(rows)
    assert p.num_tensors == 6
    assert p.num_segments == 1 + 1 + 32 + 4096 + 2048 + 3000
    assert p.segment_begin == [0, 1, 2, 34, 34 + 4096, 34 + 4096 + 2048]
    n_row_tiles = 2 + 128 + 47
    assert p.num_tiles == 7 + 1 + 4096 * 2 + n_row_tiles
    assert p.num_quant_tiles == 98 + 5 + 4096 * 20 + n_row_tiles
    assert p.num_pair_tiles == 7
    n_parts = 98 + 5 + 4096 * 20 + 32 + 2048 + 3000            # the quantize pass has the most partials
    assert p.workspace_bytes >= n_parts * 24 and p.workspace_bytes % 256 == 0
    assert qb.lib().qv2_plan_segment_begin(p.handle, 6) == -1
    p.close()
    assert (200_704 + TR - 1) // TR == 7 and (200_704 + TQ - 1) // TQ == 98 and (40000 + TQ - 1) // TQ == 20
    # without a code buffer the quantize sweep stores nothing and its tiles are as long as the read tiles
    p = qb.qv2_plan_create([_row(200_704, qrun=FAKE), _row(9408), _row(4 * 40000, qb.QV2_SYM_CHANNEL, 4),
                            _row(9408, codes=FAKE)])
    assert p.num_tiles == 7 + 1 + 4 * 2 + 1 and p.num_quant_tiles == 7 + 1 + 4 * 2 + 5
    p.close()


def test_device_calls_validate_before_touching_the_gpu():
    p = qb.qv2_plan_create([_row(1000)])
    L = qb.lib()
    ws = p.workspace_bytes
    assert L.qv2_calibrate(p.handle, None, FAKE, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_calibrate(None, FAKE, FAKE, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_calibrate(p.handle, FAKE, FAKE, FAKE, ws - 1, None) == qb.QV2_ERR_WORKSPACE
    assert L.qv2_calibrate(p.handle, FAKE, FAKE, FAKE + 4, ws, None) == qb.QV2_ERR_ALIGN
    assert L.qv2_fakequant_metrics(p.handle, FAKE, None, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_fakequant_metrics(p.handle, FAKE, FAKE, None, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_pair_metrics(p.handle, None, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_pair_metrics(p.handle, FAKE, FAKE, 0, None) == qb.QV2_ERR_WORKSPACE
    one = L.qv2_calibrate_fakequant_pair_metrics
    assert one(p.handle, None, FAKE, FAKE, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert one(p.handle, FAKE, FAKE, None, None, ws, None) == qb.QV2_ERR_NULL      # workspace
    assert one(p.handle, FAKE, FAKE, None, FAKE, ws - 1, None) == qb.QV2_ERR_WORKSPACE
    assert one(p.handle, FAKE, FAKE, FAKE + 4, FAKE, ws, None) == qb.QV2_ERR_ALIGN
    # the entry point that allocates nothing: argument checks come before any GPU call, and a
    # plan whose partial records would not fit the library's fixed array is refused
    na = L.qv2_calibrate_fakequant_pair_metrics_noalloc
    assert na(None, FAKE, FAKE, None, None) == qb.QV2_ERR_NULL
    assert na(p.handle, None, FAKE, None, None) == qb.QV2_ERR_NULL
    assert na(p.handle, FAKE, FAKE + 4, None, None) == qb.QV2_ERR_ALIGN
    assert na(p.handle, FAKE, FAKE, FAKE + 4, None) == qb.QV2_ERR_ALIGN
    big = qb.qv2_plan_create([_row(1 << 32, codes=FAKE)])           # 2 Mi quantize tiles
    assert big.workspace_bytes > qb.QV2_STATIC_SCRATCH_BYTES
    assert na(big.handle, FAKE, FAKE, None, None) == qb.QV2_ERR_WORKSPACE
    big.close()
    assert L.qv2_plan_upload(None, None) == qb.QV2_ERR_NULL
    assert L.qv2_plan_device_bytes(None) == 0 and L.qv2_plan_device_bytes(p.handle) >= 256
    whole = L.qv2_sensitivity_pass
    order = (ctypes.c_int32 * 1)()
    tail = (None, 1, None, None, None, None, order, None)
    assert whole(p.handle, FAKE, FAKE, None, FAKE, FAKE, ws, None, *tail) == qb.QV2_ERR_NULL      # d_records
    assert whole(p.handle, FAKE, FAKE, FAKE, None, FAKE, ws, None, *tail) == qb.QV2_ERR_NULL      # h_records
    assert whole(p.handle, FAKE, FAKE, FAKE + 4, FAKE, FAKE, ws, None, *tail) == qb.QV2_ERR_ALIGN
    assert whole(p.handle, FAKE, FAKE, FAKE, FAKE, FAKE, ws - 1, None, *tail) == qb.QV2_ERR_WORKSPACE
    assert whole(p.handle, FAKE, FAKE, FAKE, FAKE, FAKE, ws, None, None, 0, None, None, None, None, order,
                 None) == qb.QV2_ERR_SHAPE
    assert whole(p.handle, FAKE, FAKE, FAKE, FAKE, FAKE, ws, None, None, 1, None, None, None, None, None,
                 None) == qb.QV2_ERR_NULL                                                         # order_out


def test_binding_refuses_buffers_a_kernel_could_not_use():
    """Host tensors, short buffers, wrong element sizes and non-contiguous views never reach the
    library: the Python layer raises before any pointer is taken."""
    import torch
    host = torch.zeros(100)
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_plan_create([_row(100, x=host)])
    assert e.value.status == qb.QV2_ERR_NULL and "not a device tensor" in str(e.value)

    class FakeDev:                       # stands in for a device tensor (no GPU in this test)
        is_cuda = True

        def __init__(self, n, size=4, contiguous=True):
            self.n, self.size, self.c = n, size, contiguous

        def is_contiguous(self):
            return self.c

        def element_size(self):
            return self.size

        def numel(self):
            return self.n

        def data_ptr(self):
            return FAKE

    class FakeInt32(FakeDev):
        dtype = "torch.int32"

    for bad, what in ((dict(x=FakeDev(99)), "holds 396 bytes, 400 needed"),
                      (dict(x=FakeInt32(100)), "torch.float32 expected"),
                      (dict(x=FakeDev(100, size=8)), "8-byte elements"),
                      (dict(x=FakeDev(100, contiguous=False)), "not contiguous"),
                      (dict(qrun=FakeDev(50)), "qrun of tensor 0"),
                      (dict(codes=FakeDev(100, size=4)), "codes of tensor 0"),
                      (dict(codes=FakeDev(99, size=1)), "holds 99 bytes, 100 needed")):
        with pytest.raises(qb.QV2Error) as e:
            qb.qv2_plan_create([_row(100, **bad)])
        assert e.value.status == qb.QV2_ERR_SHAPE and what in str(e.value), str(e.value)

    p = qb.qv2_plan_create([_row(64 * 9, qb.QV2_SYM_CHANNEL, 64, x=FakeDev(64 * 9), qrun=FakeDev(64 * 9),
                                 codes=FakeDev(64 * 9, size=1))])
    ok_params, ok_sums = FakeDev(64 * 24, 1), FakeDev(64 * 32, 1)
    ws = FakeDev(p.workspace_bytes, 1)
    cases = [
        (qb.qv2_calibrate, (FakeDev(64 * 24 - 1, 1), ok_sums, ws), "d_params"),
        (qb.qv2_calibrate, (ok_params, FakeDev(63 * 32, 1), ws), "d_sums"),
        (qb.qv2_fakequant_metrics, (ok_params, host, ws), "not a device tensor"),
        (qb.qv2_pair_metrics, (FakeDev(31, 1), ws), "d_pair_sums"),
        (qb.qv2_fakequant_pair_metrics, (ok_params, ok_sums, FakeDev(8, 1), ws), "d_pair_sums"),
        (qb.qv2_calibrate_fakequant_pair_metrics, (ok_params, ok_sums, FakeDev(8, 1), ws), "d_pair_sums"),
        (qb.qv2_calibrate_fakequant_pair_metrics_cos,
         (ok_params, ok_sums, FakeDev(32, 1), FakeDev(63, 8), FakeDev(1, 8), ws), "d_seg_xxhat"),
        (qb.qv2_fakequant_pair_metrics_cos,
         (ok_params, ok_sums, FakeDev(32, 1), FakeDev(64, 8), FakeDev(0, 8), ws), "d_pair_xq"),
        (qb.qv2_tensor_sums_fold, (ok_params, ok_sums, FakeDev(47, 1)), "d_tensor_sums"),
        (qb.qv2_histogram, (ok_params, 16, FakeDev(15, 8), None, ws), "d_hist_x"),
        (qb.qv2_histogram, (ok_params, 16, FakeDev(16, 4), None, ws), "8 expected"),
    ]
    for fn, args, what in cases:
        with pytest.raises(qb.QV2Error) as e:
            fn(p, *args, stream=0)
        assert what in str(e.value), (fn.__name__, str(e.value))
    # a workspace smaller than the plan needs is the library's own check
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_calibrate(p, ok_params, ok_sums, FakeDev(p.workspace_bytes - 1, 1), stream=0)
    assert e.value.status == qb.QV2_ERR_WORKSPACE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_bn_fold(FakeDev(64 * 9 - 1), 64, 9, FakeDev(64), FakeDev(64), FakeDev(64 * 9), stream=0)
    assert "d_w" in str(e.value)
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_bn_fold(FakeDev(64 * 9), 64, 9, FakeDev(63), FakeDev(64), FakeDev(64 * 9), stream=0)
    assert "d_gamma" in str(e.value)
    p.close()


# ----------------------------------------------------------------------------
# finalize (Eq. 6-7) against the oracle on oracle-made sums
# ----------------------------------------------------------------------------
def test_finalize_matches_oracle():
    rng = np.random.default_rng(0)
    a = np.maximum(rng.standard_normal(5000) * 1.7, 0).astype(np.float32)
    w = rng.laplace(0, 0.05, (16, 27)).astype(np.float32)
    p = qb.qv2_plan_create([_row(a.size), _row(w.size, qb.QV2_SYM_CHANNEL, 16)])
    params = np.zeros(p.num_segments, qb.QPARAMS)
    sums = np.zeros(p.num_segments, qb.SUMS)
    want = []
    for t, (x, scheme, ch) in enumerate([(a, orc.ASYM_TENSOR, 1), (w, orc.SYM_CHANNEL, 16)]):
        cal = orc.calibrate(x, scheme, ch)
        fq = orc.fakequant(x, cal, scheme, ch)
        s0 = p.segment_begin[t]
        sl = slice(s0, s0 + ch)
        params["min"][sl], params["max"][sl] = cal.min, cal.max
        params["scale"][sl], params["inv_scale"][sl], params["zp"][sl] = cal.scale, cal.inv_scale, cal.zp
        sums["sum_x"][sl], sums["sum_x2"][sl], sums["sum_e2"][sl], sums["n"][sl] = \
            cal.sum_x, fq.sum_x2, fq.sum_e2, cal.n
        want.append(orc.tensor_metrics(x, cal, fq))
    got = qb.qv2_finalize(p, params, sums)
    for g, m in zip(got, want):
        assert g["mse"] == pytest.approx(m.mse, rel=1e-13)
        assert g["sqnr_db"] == pytest.approx(m.sqnr_db, abs=1e-10)
        assert g["mean"] == pytest.approx(m.mean, rel=1e-12, abs=1e-15)
        assert g["var"] == pytest.approx(m.var, rel=1e-9)
        assert g["absmax"] == np.float32(m.absmax) and g["min"] == np.float32(m.min)
        assert g["max"] == np.float32(m.max)
    # zero noise -> +inf dB; non-finite sums are reported
    sums["sum_e2"][:] = 0.0
    assert np.all(np.isinf(qb.qv2_finalize(p, params, sums)["sqnr_db"]))
    sums["sum_x2"][0] = np.nan
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_finalize(p, params, sums)
    assert e.value.status == qb.QV2_ERR_NONFINITE


def test_pair_finalize():
    rec = np.zeros(3, qb.PAIR_SUMS)
    rec["sum_ref2"], rec["sum_d2"], rec["n"] = [100.0, 4.0, 0.0], [1.0, 0.0, 0.0], [10, 4, 0]
    mse, sqnr = qb.qv2_pair_finalize(rec)
    assert mse.tolist() == [0.1, 0.0, 0.0]
    assert sqnr[0] == pytest.approx(20.0) and math.isinf(sqnr[1]) and math.isinf(sqnr[2])


# ----------------------------------------------------------------------------
# rank (Eq. 16, Algorithm 2): identical to the oracle's list
# ----------------------------------------------------------------------------
def _cfg(**kw):
    c = qb.qv2_rank_config_default()
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_rank_identical_to_oracle_random():
    rng = np.random.default_rng(21)
    for trial in range(300):
        n = int(rng.integers(1, 130))
        w = rng.uniform(10, 60, n)
        a = rng.uniform(10, 60, n)
        if trial % 3 == 0:                            # ties in the scores
            w, a = w.round(0), a.round(0)
        if trial % 7 == 0:
            w[rng.integers(0, n)] = math.inf
            a[rng.integers(0, n)] = -math.inf
        wm = rng.lognormal(0, 2.0, n)
        am = rng.lognormal(0, 2.0, n)
        if trial % 5 == 0:
            am[:] = am.round(0)                       # ties among outliers
        pos = None if trial % 2 else np.cumsum(rng.integers(1, 5, n)).astype(np.int32)
        src = trial % 3
        kw = dict(alpha_w=float(rng.uniform(0, 1)), alpha_a=float(rng.uniform(0, 1)),
                  mse_source=src, mse_factor=float(rng.choice([5.0, 2.0])))
        order, score = qb.qv2_rank(w, a, wm, am, pos, _cfg(**kw))
        o_order, o_score = orc.rank_layers(list(w), list(a), list(wm), list(am),
                                           None if pos is None else list(pos), orc.RankConfig(**kw))
        assert order.tolist() == o_order
        assert score.tolist() == o_score


def test_rank_defaults_and_optional_series():
    w = [40.0, 38.0, 45.0, 30.0, 31.0, 50.0]
    a = [30.0] * 6
    m = [1.0] * 6
    order, score = qb.qv2_rank(w, a, m, m)
    assert order.tolist() == [3, 1, 0, 4, 2, 5]
    order, _ = qb.qv2_rank(w, None, None, m)
    assert order.tolist() == [3, 1, 0, 4, 2, 5]
    order, _ = qb.qv2_rank(None, w, None, m)
    assert order.tolist() == [3, 1, 0, 4, 2, 5]


def test_rank_errors():
    w = [40.0, 38.0, 45.0]
    m = [1.0, 1.0, 1.0]
    L = qb.lib()
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank(w, w, m, [1.0, math.nan, 1.0])
    assert e.value.status == qb.QV2_ERR_NONFINITE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank(w, w, m, [1.0, -1.0, 1.0])
    assert e.value.status == qb.QV2_ERR_NONFINITE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank([1.0, math.nan, 2.0], w, m, m)
    assert e.value.status == qb.QV2_ERR_NONFINITE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank(w, w, m, m, layer_pos=[0, 2, 2])
    assert e.value.status == qb.QV2_ERR_SHAPE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank(w, w, m, None)                    # default source is the activation MSE
    assert e.value.status == qb.QV2_ERR_NULL
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank(w, w, m, m, cfg=_cfg(mse_source=3))
    assert e.value.status == qb.QV2_ERR_SHAPE
    order = np.zeros(3, np.int32)
    arr = np.array(w)
    assert L.qv2_rank(arr.ctypes.data, None, None, arr.ctypes.data, None, 0, None,
                      order.ctypes.data, None) == qb.QV2_ERR_SHAPE
    assert L.qv2_rank(None, None, None, arr.ctypes.data, None, 3, None,
                      order.ctypes.data, None) == qb.QV2_ERR_NULL
    assert L.qv2_rank(arr.ctypes.data, None, None, arr.ctypes.data, None, 3, None,
                      None, None) == qb.QV2_ERR_NULL


# ----------------------------------------------------------------------------
# baselines and BOPs cut (Sec. 7, Eq. 17): identical to the oracle
# ----------------------------------------------------------------------------
def test_bops_and_baselines_match_oracle():
    rng = np.random.default_rng(31)
    for trial in range(200):
        n = int(rng.integers(1, 130))
        macs = rng.integers(0, 10 ** 9, n).astype(np.float64)
        macs[rng.integers(0, n)] += 1.0
        w = rng.uniform(10, 60, n).round(0 if trial % 2 else 6)
        for kind in (qb.QV2_ORDER_INORDER, qb.QV2_ORDER_WEIGHT_SQNR):
            order = qb.qv2_baseline_order(kind, w)
            assert order.tolist() == orc.baseline_order(kind, list(w))
            tgt = float(rng.uniform(-5, 80))
            keep, k, pct = qb.qv2_bops_select(order, macs, tgt)
            o_keep, o_k, o_pct = orc.bops_select(order.tolist(), list(macs), tgt)
            assert keep.tolist() == o_keep and k == o_k and pct == o_pct
            assert qb.qv2_bops_reduction_pct(macs, keep) == orc.bops_reduction_pct(list(macs), o_keep)
    assert qb.qv2_baseline_order(qb.QV2_ORDER_INORDER, None, 4).tolist() == [3, 2, 1, 0]


def test_bops_errors():
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_bops_select([0, 0, 1], [1.0, 1.0, 1.0], 50.0)
    assert e.value.status == qb.QV2_ERR_SHAPE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_bops_select([0, 1], [0.0, 0.0], 50.0)
    assert e.value.status == qb.QV2_ERR_NONFINITE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_bops_select([0, 1], [1.0, -2.0], 50.0)
    assert e.value.status == qb.QV2_ERR_NONFINITE
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_baseline_order(7, [1.0, 2.0])
    assert e.value.status == qb.QV2_ERR_SCHEME
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_baseline_order(qb.QV2_ORDER_WEIGHT_SQNR, [1.0, math.nan])
    assert e.value.status == qb.QV2_ERR_NONFINITE


# ----------------------------------------------------------------------------
# histograms / KL divergence (Sec. 5, Sec. 6.1 Eq. 9): host parts
# ----------------------------------------------------------------------------
def test_kl_divergence_matches_oracle():
    rng = np.random.default_rng(41)
    for trial in range(200):
        nb = int(rng.integers(1, 300))
        p = rng.integers(0, 10 ** 6, nb).astype(np.uint64)
        q = rng.integers(0, 10 ** 6, nb).astype(np.uint64)
        p[rng.integers(0, nb)] += 1
        q[rng.integers(0, nb)] += 1
        if trial % 3 == 0:
            q[rng.integers(0, nb, max(1, nb // 4))] = 0
        for eps in (0.0, 1.0, 1e-3):
            got = qb.qv2_kl_divergence(p, q, eps)
            want = orc.kl_divergence(p.tolist(), q.tolist(), eps)
            assert got == want or got == pytest.approx(want, rel=1e-12, abs=1e-15)
    assert qb.qv2_kl_divergence([2, 2], [1, 3]) == pytest.approx(0.5 * math.log(2) + 0.5 * math.log(2 / 3))
    assert qb.qv2_kl_divergence([1, 3], [0, 4]) == math.inf
    for bad, st in (((lambda: qb.qv2_kl_divergence([0, 0], [1, 1])), qb.QV2_ERR_SHAPE),
                    ((lambda: qb.qv2_kl_divergence([1, 1], [1, 1], -1.0)), qb.QV2_ERR_NONFINITE),
                    ((lambda: qb.qv2_kl_divergence([1, 1], [1, 1, 1])), qb.QV2_ERR_SHAPE)):
        with pytest.raises(qb.QV2Error) as e:
            bad()
        assert e.value.status == st


def test_histogram_host_checks():
    p = qb.qv2_plan_create([_row(1_000_000, qrun=FAKE), _row(300)])
    assert qb.qv2_histogram_workspace_bytes(p, 1) == 0 and qb.qv2_histogram_workspace_bytes(p, 4097) == 0
    ws = qb.qv2_histogram_workspace_bytes(p, 2048)
    # 1e6 elements in chunks of at least 65536 -> 16 chunks, + 1 for the small tensor
    assert ws >= 17 * 2 * 2048 * 4 and ws % 256 == 0
    L = qb.lib()
    assert L.qv2_histogram(p.handle, FAKE, 2048, None, None, FAKE, ws, None) == qb.QV2_ERR_NULL
    assert L.qv2_histogram(p.handle, FAKE, 1, FAKE, None, FAKE, ws, None) == qb.QV2_ERR_SHAPE
    assert L.qv2_histogram(p.handle, FAKE, 2048, FAKE, None, FAKE, ws - 1, None) == qb.QV2_ERR_WORKSPACE
    assert L.qv2_histogram(p.handle, FAKE, 2048, FAKE + 4, None, FAKE, ws, None) == qb.QV2_ERR_ALIGN


def test_regroup_for_fusion_matches_oracle():
    rng = np.random.default_rng(51)
    for _ in range(300):
        n = int(rng.integers(1, 130))
        o = rng.permutation(n)
        g = rng.integers(0, max(1, n // 3), n)
        assert qb.qv2_regroup_for_fusion(o, g).tolist() == orc.regroup_for_fusion(o.tolist(), g.tolist())
    assert qb.qv2_regroup_for_fusion([4, 1, 5, 0, 3, 2], [7, 7, 8, 8, 9, 10]).tolist() == [4, 1, 0, 5, 3, 2]
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_regroup_for_fusion([0, 0, 1], [1, 1, 1])
    assert e.value.status == qb.QV2_ERR_SHAPE
    L = qb.lib()
    assert L.qv2_bn_fold(None, 4, 9, FAKE, FAKE, None, None, None, FAKE, None, None) == qb.QV2_ERR_NULL
    assert L.qv2_bn_fold(FAKE, 0, 9, FAKE, FAKE, None, None, None, FAKE, None, None) == qb.QV2_ERR_SHAPE
    assert L.qv2_bn_fold(FAKE, 4, 9, FAKE, FAKE, None, None, None, FAKE, FAKE, None) == qb.QV2_ERR_NULL


def test_rank_tensors_routes_records_to_layers():
    """qv2_rank_tensors against the manual route (finalize, scatter by layer, qv2_rank) and the
    oracle's Algorithm 2, on made-up per-tensor records; and its shape errors."""
    rng = np.random.default_rng(5)
    n_layers = 17
    rows, kinds, layers = [], [], []
    for l in rng.permutation(n_layers):            # tensors in any order
        rows.append(_row(1000 + int(l), layer=int(l), kind=0)); kinds.append(0); layers.append(int(l))
        rows.append(_row(5000 + int(l), qrun=FAKE, layer=int(l), kind=1)); kinds.append(1); layers.append(int(l))
    rows.append(_row(77, layer=3, kind=1)); kinds.append(1); layers.append(3)     # activation without a partner: ignored
    p = qb.qv2_plan_create(rows)
    nt = p.num_tensors
    ts = np.zeros(nt, qb.TENSOR_SUMS)
    ps = np.zeros(nt, qb.PAIR_SUMS)
    for t in range(nt):
        n = rows[t].numel
        ts[t] = (0.1 * n, rng.uniform(1, 4) * n, rng.uniform(1e-5, 1e-3) * n, n, -1.0, 2.0, (0, 0))
        if kinds[t] == 1 and t != nt - 1:
            f = 40.0 if layers[t] == 11 else 1.0                                   # one MSE outlier
            ps[t] = (rng.uniform(1, 4) * n, f * rng.uniform(1e-4, 2e-4) * n, n, 0)
    order, score = qb.qv2_rank_tensors(p, ts, ps, n_layers)
    met = qb.qv2_finalize_tensors(ts)
    pm, psq = qb.qv2_pair_finalize(ps)
    w_sqnr, w_mse, a_sqnr, a_mse = (np.empty(n_layers) for _ in range(4))
    for t in range(nt - 1):
        if kinds[t] == 0:
            w_sqnr[layers[t]], w_mse[layers[t]] = met["sqnr_db"][t], met["mse"][t]
        else:
            a_sqnr[layers[t]], a_mse[layers[t]] = psq[t], pm[t]
    order1, score1 = qb.qv2_rank(w_sqnr, a_sqnr, w_mse, a_mse)
    assert order.tolist() == order1.tolist() and np.array_equal(score, score1)
    o_order, _ = orc.rank_layers(list(w_sqnr), list(a_sqnr), list(w_mse), list(a_mse), None, orc.RankConfig())
    assert order.tolist() == o_order and order[0] == 11
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank_tensors(p, ts, ps, n_layers - 1)                               # layer index out of range
    assert e.value.status == qb.QV2_ERR_SHAPE
    p.close()
    # a series with a gap, and two weights in one layer
    gap = qb.qv2_plan_create([_row(10, layer=0, kind=0), _row(10, layer=1, kind=0), _row(10, qrun=FAKE, layer=0, kind=1)])
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank_tensors(gap, ts[:3], ps[:3], 2)
    assert e.value.status == qb.QV2_ERR_SHAPE
    gap.close()
    dup = qb.qv2_plan_create([_row(10, layer=0, kind=0), _row(10, layer=0, kind=0)])
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_rank_tensors(dup, ts[:2], None, 1)
    assert e.value.status == qb.QV2_ERR_SHAPE
    dup.close()
    # weights only: the activation series is left out, the rule runs on the weight MSE
    wonly = qb.qv2_plan_create([_row(10 + l, layer=l, kind=0) for l in range(5)])
    cfg = qb.qv2_rank_config_default()
    cfg.mse_source = 1
    o5, _ = qb.qv2_rank_tensors(wonly, ts[:5], None, 5, None, cfg)
    m5 = qb.qv2_finalize_tensors(ts[:5])
    o5b, _ = qb.qv2_rank(m5["sqnr_db"], None, m5["mse"], None, None, cfg)
    assert o5.tolist() == o5b.tolist()
    wonly.close()


def test_write_config_matches_oracle_text(tmp_path):
    """Sec. 4 step 5: the per-layer bit-width table, byte for byte the oracle's text; error paths."""
    rng = np.random.default_rng(9)
    n = 23
    keep = (rng.random(n) < 0.3).astype(np.uint8)
    names = [f"stage{i // 4}.conv{i % 4}" for i in range(n)]
    p1, p2 = tmp_path / "with_names.csv", tmp_path / "without.csv"
    qb.qv2_write_config(str(p1), keep, names)
    qb.qv2_write_config(str(p2), keep)
    assert p1.read_text() == orc.config_text(list(keep), names)
    assert p2.read_text() == orc.config_text(list(keep))
    assert p2.read_text().splitlines()[1] == f"0,layer0,{32 if keep[0] else 8}"
    # from a ranking: the first layers of the list are the ones at 32 bits
    order = rng.permutation(n).astype(np.int32)
    macs = rng.uniform(1e6, 1e8, n)
    flags, kept, pct = qb.qv2_bops_select(order, macs, 50.0)
    qb.qv2_write_config(str(p1), flags)
    bits = [int(l.split(",")[2]) for l in p1.read_text().splitlines()[1:]]
    assert sorted(i for i, b in enumerate(bits) if b == 32) == sorted(order[:kept].tolist())
    for bad, status in (((str(p1), keep, ["a,b"] + names[1:]), qb.QV2_ERR_SHAPE),
                        ((str(tmp_path / "no_such_dir" / "x.csv"), keep, None), qb.QV2_ERR_IO)):
        with pytest.raises(qb.QV2Error) as e:
            qb.qv2_write_config(*bad)
        assert e.value.status == status
    assert qb.lib().qv2_write_config(None, keep.ctypes.data, None, n) == qb.QV2_ERR_NULL
    assert qb.lib().qv2_write_config(str(p1).encode(), keep.ctypes.data, None, 0) == qb.QV2_ERR_SHAPE
