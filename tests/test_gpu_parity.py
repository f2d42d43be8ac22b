"""GPU parity: the HIP library (through the C ABI) against the CPU oracle,
element by element, on seeded synthetic tensor sets with the paper's model
shapes plus the edge cases of the method."""
import numpy as np
import pytest
import torch

import harness as H
from oracle import reference as orc
from paper_2501_07161_amd import binding as qb
from paper_2501_07161_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
A, S, C = qb.QV2_ASYM_TENSOR, qb.QV2_SYM_TENSOR, qb.QV2_SYM_CHANNEL


def _run_config(specs, rank_kwargs=None, fused=False):
    items = H.items_from_specs(specs, DEV)
    H.attach_pairs(items, specs)
    res = H.run_gpu(items, fused=fused)
    rows = H.check_all(items, res)
    order = H.check_ranking(items, res, rows, rank_kwargs)
    return items, res, order


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_config_tiny(fused):
    """Three tensors, per-tensor asymmetric: conv weight, ReLU activation with a pair, fc weight."""
    items, res, order = _run_config(synth.config_tiny(), fused=fused)
    assert res.plan.num_segments == 3 and sorted(order) == [0, 1]
    # the activation is post-ReLU: min 0, zero-point at the bottom code
    assert res.params["min"][1] == 0.0 and res.params["zp"][1] == -128


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_config_resnet18_batch32(fused):
    """ResNet-18 shapes at the stated batch: 21 weights + 21 activations, per-tensor asymmetric."""
    items, res, order = _run_config(synth.config_resnet18(32), fused=fused)
    assert len(order) == 21 and sorted(order) == list(range(21))


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_config_mobilenetv2_per_channel(fused):
    """MobileNetV2 shapes: per-output-channel symmetric weights with rows of 9 / 27 / ...
    elements, Laplace + outlier values, ReLU6 activations (batch reduced so the oracle stays fast)."""
    items, res, order = _run_config(synth.config_mobilenetv2(8), fused=fused)
    assert len(order) == 53
    dw = [t for t, it in enumerate(items) if it.name.endswith(".dw.w")]
    assert dw and all(items[t].x.numel() // items[t].channels == 9 for t in dw)


@pytest.mark.parametrize("per_channel", [False, True])
def test_config_vgg16_weights_full_size(per_channel):
    """All VGG-16 weights at full size (fc6 = 102.8M elements; per-channel rows of 25088
    elements are one stream tile each); activations at batch 2."""
    _run_config(synth.config_vgg16(2, per_channel))


@pytest.mark.parametrize("bnfold,fused", [(False, False), (True, False), (True, True), (False, "single")])
def test_config_resnet50_small_batch(bnfold, fused):
    """ResNet-50 shapes, per-channel weights (plain and BN-folded variants), batch 4."""
    items, res, order = _run_config(synth.config_resnet50(4, bnfold), fused=fused)
    assert len(order) == 54


# ----------------------------------------------------------------------------
# edge cases
# ----------------------------------------------------------------------------
def _rand(n, seed, scale=1.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return torch.randn(n, generator=g, device=DEV) * scale


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_ragged_lengths_and_unaligned_pointers(fused):
    """Lengths around tile and vector boundaries, inputs starting 4 / 8 / 12 bytes past a
    16-byte boundary, code buffers starting 1..3 bytes past a 4-byte boundary."""
    items = []
    lens = [1, 2, 3, 4, 5, 7, 63, 64, 65, 255, 1023, 1025, 4099, 16383, 16384, 16385, 16387,
            2047, 2048, 2049, 4095, 4096, 4097, 8195, 32767, 32768, 32769, 65536 + 5, 100_003]
    for i, n in enumerate(lens):
        for off in range(4):
            base = _rand(n + 8, 100 + i)
            x = base[off: off + n]
            scheme = A if (i + off) % 2 == 0 else S
            q = (x + 0.01 * _rand(n + 4, 900 + i)[off: off + n]) if off % 2 == 0 else None
            # a pair whose two tensors have different offsets inside 16 bytes
            if off == 3:
                q = (_rand(n + 8, 500 + i)[1: 1 + n])
            items.append(H.Item(f"len{n}.off{off}", x, scheme, 1, 1, len(items), qrun=q,
                                codes_offset=(i + off) % 4))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_per_channel_row_shapes(fused):
    """Rows of 1, 3, 9, 27, 64, 65, 576, 8191, 8192 (LDS row groups) and 8193, 20001, 40000,
    70001 (rows as one or several stream tiles, unaligned row starts), with unaligned bases and
    code buffers."""
    items = []
    shapes = [(7, 1), (5000, 1), (33, 3), (960, 9), (1100, 9), (64, 27), (10, 64), (10, 65),
              (37, 576), (3, 8191), (5, 8192), (3, 8193), (4, 20001), (1, 17), (2, 40000), (3, 70001)]
    for i, (c, inner) in enumerate(shapes):
        for off in (0, 1):
            base = _rand(c * inner + 4, 200 + i, 0.1)
            x = base[off: off + c * inner]
            if i % 3 == 0:
                x.view(c, inner)[c // 2] = 0.0          # a dead channel
            q = (x * 0.97 + 0.001) if i % 2 == 0 else None     # a quantized-run partner of a weight
            items.append(H.Item(f"rows{c}x{inner}.off{off}", x, C, c, 0, len(items), qrun=q,
                                codes_offset=(i + off) % 4))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_per_channel_rows_held_in_registers(fused):
    """Rows of a multiple of 4 elements (64 ... 8192) on 16-byte boundaries with 4-byte aligned
    code buffers take the register form of the row kernels: 16 to 128 lanes per row, last vectors
    only partly populated (68, 100, 1028, 4100, 8188), tiles whose last workgroup has fewer rows
    than lanes groups, with and without partners, dead channels."""
    items = []
    shapes = [(9, 64), (7, 68), (5, 100), (33, 256), (600, 128), (3, 1020), (4, 1024), (6, 1028),
              (35, 1024), (3, 4096), (2, 4100), (5, 4608), (3, 8188), (2, 8192), (1, 8192)]
    for i, (c, inner) in enumerate(shapes):
        x = _rand(c * inner, 800 + i, 0.1)
        if i % 4 == 0:
            x.view(c, inner)[c // 2] = 0.0
        q = (x * 1.02 - 0.0005) if i % 2 == 0 else None
        items.append(H.Item(f"reg{c}x{inner}", x, C, c, 0, len(items), qrun=q))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_long_per_channel_rows_held_in_registers(fused):
    """Rows beyond what the LDS copy holds: 8196 ... 16384 elements take one row per 256-thread
    workgroup, 16388 ... 32768 (the 25088 of VGG-16's first fully connected layer among them)
    one row per 512-thread workgroup; 32772 is a stream row again.  With and without partners,
    last vectors partly populated, a dead channel; plus the same lengths where the register form
    does not apply (base 4 bytes off a 16-byte boundary, code buffer 1 byte off)."""
    items = []
    shapes = [(3, 8196), (5, 12288), (2, 16384), (3, 16388), (4, 25088), (2, 32764), (2, 32768), (2, 32772)]
    for i, (c, inner) in enumerate(shapes):
        x = _rand(c * inner, 850 + i, 0.1)
        if i % 3 == 0:
            x.view(c, inner)[c // 2] = 0.0
        q = (x * 0.98 + 0.0007) if i % 2 == 0 else None
        items.append(H.Item(f"long{c}x{inner}", x, C, c, 0, len(items), qrun=q))
    for i, (c, inner) in enumerate([(2, 12288), (2, 25088)]):
        base = _rand(c * inner + 4, 870 + i, 0.1)
        items.append(H.Item(f"long{c}x{inner}.off1", base[1: 1 + c * inner], C, c, 0, len(items)))
        items.append(H.Item(f"long{c}x{inner}.codes1", _rand(c * inner, 880 + i, 0.1), C, c, 0, len(items),
                            codes_offset=1))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)
    # the forms the plan chose: 256-thread rows, 512-thread rows, stream tiles
    once = [qb.qv2_plan_create([qb.TensorArg(x=it.x, numel=it.x.numel(), scheme=C, channels=it.channels,
                                             codes=it.codes)]).num_single_read_elements > 0 for it in items]
    assert once == [True] * 7 + [False] + [False] * 4


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_degenerate_and_special_values(fused):
    z = torch.zeros(5000, device=DEV)
    const = torch.full((4097,), 3.25, device=DEV)
    neg = -torch.rand(9000, device=DEV) - 0.5
    negzero = torch.zeros(100, device=DEV)
    negzero[::2] = -0.0
    tiny = torch.full((300,), 1e-42, device=DEV)           # sub-normal range -> degenerate step
    grid = ((torch.arange(-128, 128, device=DEV, dtype=torch.float32) + 3) * 0.0625).repeat(70)
    big = _rand(20000, 7, 1e30)
    small = _rand(20000, 8, 1e-30)
    one = torch.tensor([-2.5], device=DEV)
    items = []
    for name, x in [("zeros", z), ("const", const), ("neg", neg), ("negzero", negzero),
                    ("tiny", tiny), ("grid", grid), ("big", big), ("small", small), ("one", one)]:
        for scheme in (A, S):
            items.append(H.Item(f"{name}.{scheme}", x, scheme, 1, 0, len(items), qrun=x.clone()))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)
    t = [i for i, it in enumerate(items) if it.name == "grid.0"][0]
    assert res.metrics[t]["mse"] == 0.0 and np.isinf(res.metrics[t]["sqnr_db"])   # int8-grid fact
    assert np.all(res.pair["sum_d2"] == 0.0) and np.all(np.isinf(res.pair_sqnr))   # identical pairs


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_many_small_tiles(fused, monkeypatch):
    """Tile lengths forced down to 512 / 256 elements (tuning knobs read when a plan is made):
    medium tensors then span hundreds to thousands of tiles, so the one-wavefront and the
    whole-workgroup folds, ragged last tiles and per-channel rows cut into several tiles are all
    exercised on inputs the oracle still finishes in seconds."""
    monkeypatch.setenv("QV2_TILE_ELEMS", "512")
    monkeypatch.setenv("QV2_QUANT_TILE_ELEMS", "256")
    items = []
    for i, n in enumerate([1, 255, 256, 257, 511, 513, 9_999, 65_537, 300_001, 1_000_003]):
        x = _rand(n + 4, 600 + i)[i % 4: i % 4 + n]
        q = x * 0.99 + 0.002 if i % 3 != 1 else None
        items.append(H.Item(f"t{n}", x, A if i % 2 else S, 1, 1, len(items), qrun=q, codes_offset=i % 4))
    for i, (c, inner) in enumerate([(3, 8193), (5, 20_001), (2, 70_001), (40, 300)]):
        x = _rand(c * inner + 4, 700 + i, 0.2)[1: 1 + c * inner]
        items.append(H.Item(f"rows{c}x{inner}", x, C, c, 0, len(items), qrun=x * 1.01 if i % 2 == 0 else None))
    res = H.run_gpu(items, fused=fused)
    assert res.plan.num_quant_tiles > 6000
    H.check_all(items, res)


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16, 17, 18])
def test_random_layer_tables(seed):
    """Randomly drawn layer tables: sizes from 1 to 300 K elements, any scheme, channel counts and
    row lengths on both sides of every path's limits (LDS rows, register rows, rows as stream
    tiles), bases and code buffers at random offsets, partners present, absent or misaligned against
    x, some tensors without code buffers.  Every call form against the oracle."""
    rng = np.random.default_rng(seed)
    items = []
    for i in range(28):
        kind = int(rng.integers(0, 4))
        if kind == 0:
            c, inner = 1, int(rng.integers(1, 300_000))
            scheme = A if rng.random() < 0.5 else S
        elif kind == 1:                      # short rows
            c, inner = int(rng.integers(1, 400)), int(rng.integers(1, 130))
            scheme = C
        elif kind == 2:                      # rows around the register / LDS forms
            inner = int(rng.choice([64, 128, 132, 576, 1000, 1024, 2048, 4100, 4608, 8188, 8192])) + int(rng.choice([0, 0, 0, 1, 3]))
            c, scheme = int(rng.integers(1, 12)), C
        else:                                # rows longer than the row-group limit
            c, inner, scheme = int(rng.integers(1, 5)), int(rng.integers(8193, 60_000)), C
        n = c * inner
        off = int(rng.choice([0, 0, 0, 1, 2, 3]))
        x = _rand(n + 8, 1000 * seed + i, float(rng.choice([1e-3, 0.1, 1.0, 30.0])))[off: off + n]
        if rng.random() < 0.3:
            x = x.clamp(min=0)
        r = rng.random()
        if r < 0.4:
            q = None
        elif r < 0.85:
            q = _rand(n + 8, 5000 * seed + i, 0.01)[off: off + n] + x
        else:                                # partner at another offset inside 16 bytes
            qo = (off + 1 + int(rng.integers(0, 3))) % 4
            q = _rand(n + 8, 5000 * seed + i, 0.01)[qo: qo + n] + x
        items.append(H.Item(f"r{i}.{c}x{inner}.off{off}", x, scheme, c, int(rng.integers(0, 2)), len(items), qrun=q,
                            want_codes=bool(rng.random() < 0.85), codes_offset=int(rng.choice([0, 0, 1, 2, 3]))))
    for form in (False, True, "single"):
        res = H.run_gpu(items, fused=form)
        H.check_all(items, res)


@pytest.mark.parametrize("fused", [False, "single"])
def test_thousands_of_tensors(fused):
    """A layer table of 3000 tensors, most of them a fraction of one tile, a few long ones in
    between: the table from tile index to tensor then has fewer entries than there are tensors,
    so finding a tile walks over several records, and the fold launches see thousands of one-record
    segments."""
    rng = np.random.default_rng(77)
    items = []
    for i in range(3000):
        r = rng.random()
        if i % 750 == 400:
            c, inner, scheme = 1, 150_001 + i, A
        elif r < 0.6:
            c, inner, scheme = 1, int(rng.integers(1, 2500)), (A if rng.random() < 0.5 else S)
        elif r < 0.9:
            c, inner, scheme = int(rng.integers(1, 9)), int(rng.integers(1, 200)), C
        else:
            c, inner, scheme = int(rng.integers(1, 4)), int(rng.choice([64, 128, 576, 1024])), C
        n = c * inner
        x = _rand(n, 90_000 + i, float(rng.choice([0.05, 1.0, 8.0])))
        q = x * 0.98 + 0.001 if rng.random() < 0.5 else None
        items.append(H.Item(f"n{i}.{c}x{inner}", x, scheme, c, int(rng.integers(0, 2)), len(items), qrun=q,
                            want_codes=bool(rng.random() < 0.9)))
    res = H.run_gpu(items, fused=fused)
    assert res.plan.num_tensors == 3000
    H.check_all(items, res)


def test_cached_params_clip_both_ends():
    """Parameters handed in by the caller (the calibration cache) instead of calibrating:
    a range narrower than the data saturates codes at -128 and 127."""
    x = _rand(50_000, 11, 2.0)
    w = _rand(64 * 100, 12, 0.3)
    items = [H.Item("x", x, A, 1, 1, 0), H.Item("w", w, C, 64, 0, 1)]
    params = np.zeros(65, qb.QPARAMS)
    sc, inv, zp = orc.params(-1.0, 2.0, orc.ASYM_TENSOR)
    params[0] = (-1.0, 2.0, sc, inv, zp, 0)
    for c in range(64):
        sc, inv, zp = orc.params(-0.01 * (c + 1), 0.01 * (c + 1), orc.SYM_CHANNEL)
        params[1 + c] = (-0.01 * (c + 1), 0.01 * (c + 1), sc, inv, zp, 0)
    res = H.run_gpu(items, params_override=params)
    for t, it in enumerate(items):
        xh = it.x.cpu().numpy().reshape(-1)
        s0 = res.plan.segment_begin[t]
        S_ = it.channels
        cal = orc.Calibration(params["min"][s0:s0 + S_], params["max"][s0:s0 + S_],
                              params["scale"][s0:s0 + S_], params["inv_scale"][s0:s0 + S_],
                              params["zp"][s0:s0 + S_], None, None,
                              np.full(S_, xh.size // S_, np.int64))
        fq = orc.fakequant(xh, cal, it.scheme, it.channels)
        got = it.codes.cpu().numpy()
        assert np.array_equal(got, fq.codes)
        assert got.min() == -128 and got.max() == 127
        U = res.sums[s0:s0 + S_]
        assert np.all(np.abs(U["sum_e2"] - fq.sum_e2) <= H.MSE_RTOL * fq.sum_e2)
        assert np.all(np.abs(U["sum_x2"] - fq.sum_x2) <= H.SX2_RTOL * fq.sum_x2)


def test_metrics_only_without_code_buffers():
    x = _rand(70_001, 13)
    w = _rand(48 * 27, 14, 0.1)
    with_codes = [H.Item("x", x, A), H.Item("w", w, C, 48)]
    without = [H.Item("x", x, A, want_codes=False), H.Item("w", w, C, 48, want_codes=False)]
    r1, r2 = H.run_gpu(with_codes), H.run_gpu(without)
    assert r1.sums.tobytes() == r2.sums.tobytes() and r1.params.tobytes() == r2.params.tobytes()


def test_bit_stable_across_runs():
    specs = synth.config_resnet50(2)
    items = H.items_from_specs(specs, DEV)
    for it in items:
        if it.kind == synth.ACTIVATION:
            it.qrun = it.x + 0.01
    r1 = H.run_gpu(items)
    c1 = [it.codes.clone() for it in items]
    r2 = H.run_gpu(items)
    assert r1.params.tobytes() == r2.params.tobytes()
    assert r1.sums.tobytes() == r2.sums.tobytes()
    assert r1.pair.tobytes() == r2.pair.tobytes()
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))


def test_fused_call_equals_the_two_separate_calls():
    """qv2_fakequant_pair_metrics against qv2_fakequant_metrics + qv2_pair_metrics: codes and
    the per-segment sums bit-identical; pair sums equal up to fp64 summation order."""
    specs = synth.config_resnet50(2)
    items = H.items_from_specs(specs, DEV)
    for it in items:
        if it.kind == synth.ACTIVATION:
            it.qrun = it.x * 0.98 + 0.003
    r1 = H.run_gpu(items)
    c1 = [it.codes.clone() for it in items]
    r2 = H.run_gpu(items, fused=True)
    assert r1.params.tobytes() == r2.params.tobytes()
    assert r1.sums.tobytes() == r2.sums.tobytes()
    assert np.array_equal(r1.pair["n"], r2.pair["n"])
    for f in ("sum_ref2", "sum_d2"):
        assert np.allclose(r1.pair[f], r2.pair[f], rtol=1e-12, atol=0)
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))


def test_single_call_pass_equals_the_separate_calls():
    """qv2_calibrate_fakequant_pair_metrics (row-group tensors read from HBM once) against
    qv2_calibrate + qv2_fakequant_pair_metrics: parameters, codes, sum x and sum e^2 equal bit for
    bit, sum x^2 and the pair sums up to fp64 summation order; without pair sums it equals qv2_calibrate +
    qv2_fakequant_metrics."""
    specs = synth.config_mobilenetv2(2) + synth.config_resnet50(2) + synth.config_tiny()
    items = H.items_from_specs(specs, DEV)
    for i, it in enumerate(items):
        if it.kind == synth.ACTIVATION or i % 5 == 0:       # some weights get a partner too
            it.qrun = it.x * 0.98 + 0.003
    items.append(H.Item("rows.unaligned", _rand(960 * 9 + 4, 77, 0.1)[1: 1 + 960 * 9], C, 960, 0, 0,
                        qrun=_rand(960 * 9 + 4, 78, 0.1)[3: 3 + 960 * 9], codes_offset=3))
    r1 = H.run_gpu(items, fused=True)
    c1 = [it.codes.clone() for it in items]
    r2 = H.run_gpu(items, fused="single")
    assert r2.plan.num_tiles > r2.plan.num_tensors          # row-group and stream tiles both present
    assert r1.params.tobytes() == r2.params.tobytes()
    H.same_sums_single_call(r2.sums, r1.sums)
    assert np.array_equal(r1.pair["n"], r2.pair["n"])
    for f in ("sum_ref2", "sum_d2"):        # taken in the calibration sweep: other tile lengths
        assert np.allclose(r1.pair[f], r2.pair[f], rtol=1e-12, atol=0)
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))
    # no pair sums: the plain fake-quant results
    r3 = H.run_gpu(items)
    buf = qb.Buffers(r3.plan, torch.device(DEV))
    for it in items:
        it.codes.fill_(0x55)
    qb.qv2_calibrate_fakequant_pair_metrics(r3.plan, buf.params, buf.sums, None, buf.workspace)
    torch.cuda.synchronize()
    params, sums, _ = buf.host()
    assert params.tobytes() == r3.params.tobytes()
    H.same_sums_single_call(sums, r3.sums)
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))


def test_cosine_similarity_variant():
    """qv2_fakequant_pair_metrics_cos: cos(x, xhat) and cos(x, qrun) against the oracle's direct
    definition; every other output bit-identical to the call without the cross terms."""
    specs = synth.config_mobilenetv2(4) + synth.config_tiny()
    items = H.items_from_specs(specs, DEV)
    H.attach_pairs(items, specs)
    extra = [H.Item("zeros", torch.zeros(5000, device=DEV), A, qrun=torch.zeros(5000, device=DEV)),
             H.Item("zero_q", _rand(5000, 31), S, qrun=torch.zeros(5000, device=DEV)),
             H.Item("big", _rand(30_001, 32, 1e25)[1:], A, qrun=_rand(30_000, 33, 1e25)),
             H.Item("rows_q", _rand(64 * 27, 34, 0.1), C, 64, qrun=_rand(64 * 27, 35, 0.1)),
             H.Item("neg_q", _rand(70_000, 36), A, qrun=-_rand(70_000, 36))]
    for it in extra:
        it._oracle = None
    items += extra
    r1 = H.run_gpu(items, fused=True)
    c1 = [it.codes.clone() for it in items]
    r2 = H.run_gpu(items, cos=True)
    H.check_all(items, r2)
    assert r1.sums.tobytes() == r2.sums.tobytes() and r1.pair.tobytes() == r2.pair.tobytes()
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))
    # the single call with the cross terms: same cosines, against the oracle again
    r3 = H.run_gpu(items, fused="single", cos=True)
    H.check_all(items, r3)
    assert r3.params.tobytes() == r2.params.tobytes()
    H.same_sums_single_call(r3.sums, r2.sums)
    assert np.allclose(r3.cos_quant, r2.cos_quant, rtol=0, atol=1e-12, equal_nan=True)
    assert np.allclose(r3.cos_pair, r2.cos_pair, rtol=0, atol=1e-12, equal_nan=True)
    assert all(torch.equal(a, it.codes) for a, it in zip(c1, items))
    names = [it.name for it in items]
    assert r2.cos_quant[names.index("zeros")] == 1.0 and r2.cos_pair[names.index("zeros")] == 1.0
    assert r2.cos_pair[names.index("zero_q")] == 0.0
    assert abs(r2.cos_pair[names.index("neg_q")] + 1.0) < 1e-12


@pytest.mark.parametrize("nbins", [7, 2048, 4096])
def test_histograms_and_kl_divergence(nbins):
    """qv2_histogram: counts bit-exact against the oracle (same fp32 binning rule) for x and for
    qrun over x's calibrated range; KL divergence from those counts."""
    specs = synth.config_tiny() + synth.config_mobilenetv2(2)
    items = H.items_from_specs(specs, DEV)
    H.attach_pairs(items, specs)
    items += [H.Item("ragged", _rand(200_003, 51)[3:], A, qrun=_rand(200_001, 52)[1:] * 3.0),   # qrun wider than x
              H.Item("zeros", torch.zeros(70_000, device=DEV), A, qrun=torch.zeros(70_000, device=DEV)),
              H.Item("rows", _rand(48 * 27, 53, 0.1), C, 48, qrun=_rand(48 * 27, 54, 0.1)),
              H.Item("long", torch.relu(_rand(1_500_000, 55)), A, qrun=torch.relu(_rand(1_500_000, 55)) + 0.01)]
    res = H.run_gpu(items, fused=True)
    plan, buf = res.plan, res.buffers
    hx = torch.zeros(plan.num_tensors * nbins, dtype=torch.int64, device=DEV)
    hq = torch.ones(plan.num_tensors * nbins, dtype=torch.int64, device=DEV)
    ws = torch.zeros(qb.qv2_histogram_workspace_bytes(plan, nbins), dtype=torch.uint8, device=DEV)
    qb.qv2_histogram(plan, buf.params, nbins, hx, hq, ws)
    torch.cuda.synchronize()
    hx = hx.cpu().numpy().astype(np.uint64).reshape(plan.num_tensors, nbins)
    hq = hq.cpu().numpy().astype(np.uint64).reshape(plan.num_tensors, nbins)
    for t, it in enumerate(items):
        x = it.x.cpu().numpy().reshape(-1)
        lo, hi = np.float32(x.min()) + np.float32(0), np.float32(x.max()) + np.float32(0)
        want = orc.histogram(x, lo, hi, nbins)
        assert np.array_equal(hx[t], want), f"{it.name}: x histogram"
        assert int(hx[t].sum()) == x.size
        if it.qrun is None:
            assert not hq[t].any()
            continue
        wq = orc.histogram(it.qrun.cpu().numpy().reshape(-1), lo, hi, nbins)
        assert np.array_equal(hq[t], wq), f"{it.name}: qrun histogram"
        for eps in (0.0, 1.0):
            got, ref = qb.qv2_kl_divergence(hx[t], hq[t], eps), orc.kl_divergence(want.tolist(), wq.tolist(), eps)
            assert got == ref or abs(got - ref) <= 1e-12 * abs(ref) + 1e-15, f"{it.name}: KL"
    assert qb.qv2_kl_divergence(hx[-3], hq[-3], 0.0) == 0.0        # identical (all-zero) tensors


def test_bn_fold_bit_exact():
    """Eq. 12 on the device against the oracle: folded weights and bias bit-exact; folding in
    place; then the folded weight goes through the pass like any other tensor."""
    g = torch.Generator(device=DEV)
    g.manual_seed(61)
    for ch, inner in ((64, 147), (7, 1), (3, 100_003), (512, 4608)):
        w = torch.randn(ch, inner, generator=g, device=DEV)
        gamma = torch.rand(ch, generator=g, device=DEV) + 0.5
        var = torch.rand(ch, generator=g, device=DEV) * 3 + 0.05
        mean, beta, bias = (torch.randn(ch, generator=g, device=DEV) for _ in range(3))
        w_out, b_out = torch.empty_like(w), torch.empty(ch, device=DEV)
        qb.qv2_bn_fold(w, ch, inner, gamma, var, w_out, bias, mean, beta, b_out)
        torch.cuda.synchronize()
        a, c = orc.bn_fold(w.cpu().numpy(), gamma.cpu().numpy(), var.cpu().numpy(), mean.cpu().numpy(),
                           beta.cpu().numpy(), bias.cpu().numpy())
        assert np.array_equal(w_out.cpu().numpy().view(np.uint32), a.view(np.uint32))
        assert np.array_equal(b_out.cpu().numpy().view(np.uint32), c.view(np.uint32))
        w2 = w.clone()
        qb.qv2_bn_fold(w2, ch, inner, gamma, var, w2)                     # in place, no bias
        torch.cuda.synchronize()
        assert torch.equal(w2, w_out)
    it = H.Item("folded", w_out, C, 512)
    H.check_all([it], H.run_gpu([it]))


def test_cross_kernel_pair_of_dequantized_equals_fakequant_error():
    """pair(x, dequant(codes)) must reproduce the fake-quant pass's own noise energy."""
    x = torch.relu(_rand(300_000, 15, 1.5))
    it = H.Item("x", x, A)
    r = H.run_gpu([it])
    sc, zp = float(r.params["scale"][0]), int(r.params["zp"][0])
    xhat = torch.from_numpy(orc.dequantize(it.codes.cpu().numpy(), sc, zp)).to(DEV)
    it2 = H.Item("x", x, A, qrun=xhat)
    r2 = H.run_gpu([it2])
    assert abs(r2.pair["sum_d2"][0] - r.sums["sum_e2"][0]) <= 1e-9 * r.sums["sum_e2"][0]
    assert abs(r2.pair["sum_ref2"][0] - r.sums["sum_x2"][0]) <= 1e-9 * r.sums["sum_x2"][0]


def test_non_default_stream():
    x = _rand(123_457, 16)
    s = torch.cuda.Stream()
    it = H.Item("x", x, A, qrun=x * 0.99)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        res = H.run_gpu([it])
    H.check_all([it], res)


def test_device_calls_can_be_captured_in_a_graph():
    """The device part of the pass (single call + per-tensor fold) captured in a HIP graph through
    torch and replayed three times, with eager work and synchronisations in between: every replay
    reproduces the eager records and codes bit for bit.  (The plan's tables are uploaded by the
    eager call before the capture; the calls record no memset nodes and never synchronise.)"""
    specs = synth.config_mobilenetv2(2) + synth.config_tiny()
    items = H.items_from_specs(specs, DEV)
    for it in items:
        if it.kind == synth.ACTIVATION:
            it.qrun = it.x * 0.98 + 0.003
    res = H.run_gpu(items, fused="single")
    plan, buf = res.plan, res.buffers
    dev = torch.device(DEV)
    tsums = torch.zeros(plan.num_tensors * qb.TENSOR_SUMS.itemsize, dtype=torch.uint8, device=dev)

    def device_part():
        qb.qv2_calibrate_fakequant_pair_metrics(plan, buf.params, buf.sums, buf.pair, buf.workspace)
        qb.qv2_tensor_sums_fold(plan, buf.params, buf.sums, tsums)

    device_part()
    torch.cuda.synchronize()
    want = [buf.params.clone(), buf.sums.clone(), buf.pair.clone(), tsums.clone()] + [it.codes.clone() for it in items]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        device_part()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        device_part()
    for rep in range(3):
        for t in (buf.params, buf.sums, buf.pair, tsums, buf.workspace):
            t.fill_(0x5A)                                   # eager work between the replays
        for it in items:
            it.codes.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [buf.params, buf.sums, buf.pair, tsums] + [it.codes for it in items]
        assert all(torch.equal(a, b) for a, b in zip(got, want)), f"replay {rep}"


# ----------------------------------------------------------------------------
# what the header promises beyond finite inputs and one call at a time
# ----------------------------------------------------------------------------
def _poisoned_set():
    """Two layers, each a weight and an activation with a partner, plus a lone activation and a
    per-channel weight.  NaN and +-Inf entries sit at a tensor's first element, inside the vector
    body, in the scalar tail and in single channels."""
    nan, inf = float("nan"), float("inf")
    w0 = _rand(9408, 301, 0.05)
    a0 = torch.relu(_rand(200_707, 302))
    a0[0] = nan; a0[70_001] = nan; a0[-1] = nan
    w1 = _rand(640, 303, 0.1)
    w1[5] = inf; w1[333] = -inf
    a1 = torch.relu(_rand(50_176, 304))
    lone = _rand(33_001, 305)                        # no partner: takes no part in the ranking
    lone[12_345] = nan
    pc = _rand(64 * 576, 306, 0.1)                   # 64 channels in the row kernels
    pc.view(64, 576)[3, 7] = nan
    pc.view(64, 576)[40, 0] = inf
    pl = _rand(6 * 20_001, 307, 0.1)                 # 6 channels as stream tiles
    pl.view(6, 20_001)[2, 19_999] = nan
    items = [H.Item("w0", w0, A, 1, synth.WEIGHT, 0), H.Item("a0.nan", a0, A, 1, synth.ACTIVATION, 0, qrun=a0 * 0.99),
             H.Item("w1.inf", w1, S, 1, synth.WEIGHT, 1), H.Item("a1", a1, A, 1, synth.ACTIVATION, 1, qrun=a1 * 0.98 + 0.01),
             H.Item("lone.nan", lone, A, 1, synth.ACTIVATION, 2), H.Item("pc.rows", pc, C, 64, synth.ACTIVATION, 3),
             H.Item("pc.long", pl, C, 6, synth.ACTIVATION, 4)]
    return items


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_nan_and_inf_inputs(fused):
    """Inputs must be finite; what happens otherwise is still defined: NaNs are ignored by min / max
    and poison the sums of their own segment only; finalize reports ERR_NONFINITE and still writes
    every metric.  Range and n against the oracle for every tensor, everything for the clean ones."""
    items = _poisoned_set()
    res = H.run_gpu(items, fused=fused)
    for t, it in enumerate(items):
        x = it.x.cpu().numpy().reshape(-1)
        cal = orc.calibrate(x, it.scheme, it.channels)
        s0 = res.plan.segment_begin[t]
        n_seg = it.channels if it.scheme == C else 1
        P, U = res.params[s0:s0 + n_seg], res.sums[s0:s0 + n_seg]
        assert np.array_equal(P["min"].view(np.uint32), cal.min.view(np.uint32)), it.name
        assert np.array_equal(P["max"].view(np.uint32), cal.max.view(np.uint32)), it.name
        assert np.array_equal(U["n"], cal.n), it.name
        seg = x.reshape(n_seg, -1)
        dirty = ~np.isfinite(seg).all(axis=1)
        assert np.all(~np.isfinite(U["sum_x2"][dirty]) | ~np.isfinite(U["sum_e2"][dirty])), it.name
        clean = np.nonzero(~dirty)[0]
        fq = orc.fakequant(x, cal, it.scheme, it.channels)
        assert np.array_equal(P["scale"][clean].view(np.uint32), cal.scale[clean].view(np.uint32)), it.name
        assert np.array_equal(P["zp"][clean], cal.zp[clean]), it.name
        assert np.all(np.abs(U["sum_e2"][clean] - fq.sum_e2[clean]) <= H.MSE_RTOL * fq.sum_e2[clean]), it.name
        assert np.all(np.abs(U["sum_x2"][clean] - fq.sum_x2[clean]) <= H.SX2_RTOL * fq.sum_x2[clean]), it.name
        codes = it.codes.cpu().numpy().reshape(n_seg, -1)
        assert np.array_equal(codes[clean], fq.codes.reshape(n_seg, -1)[clean]), it.name
        if not dirty.any():
            H.check_item(t, it, res)
    # the host half says so, and writes every record anyway
    with pytest.raises(qb.QV2Error) as e:
        qb.qv2_finalize(res.plan, res.params, res.sums)
    assert e.value.status == qb.QV2_ERR_NONFINITE
    assert np.isfinite(res.metrics["mse"][[0, 3]]).all() and np.isnan(res.metrics["mse"][1])
    assert np.isnan(res.pair_mse[1]) and np.isfinite(res.pair_mse[3])


def test_sensitivity_pass_reports_nonfinite_after_writing_every_output():
    """One native call over a set with NaN / Inf entries: ERR_NONFINITE, every metric written.  With
    the bad values outside the series the ranking uses the list is the true one; with a NaN SQNR
    inside them no list can be made and the outputs hold layer order and NaN scores."""
    def run(items):
        res = H.run_gpu(items, fused="single")
        n_layers = max(it.layer for it in items) + 1
        buf = qb.Buffers(res.plan, DEV)
        out = qb.PassOutputs(res.plan, n_layers, DEV)
        out.order[:] = -7
        out.score[:] = -7.0
        with pytest.raises(qb.QV2Error) as e:
            qb.qv2_sensitivity_pass(res.plan, buf.params, buf.sums, out, buf.workspace)
        assert e.value.status == qb.QV2_ERR_NONFINITE
        assert np.array_equal(out.metrics["mse"], res.metrics["mse"], equal_nan=True)
        assert np.array_equal(out.pair_mse, res.pair_mse, equal_nan=True)
        return res, out

    # (1) only the lone activation (no partner, so in no series) is poisoned: the list is the true one
    items = [it for it in _poisoned_set()[:5]]
    items[1] = H.Item("a0", torch.relu(_rand(200_707, 302)), A, 1, synth.ACTIVATION, 0)
    items[1].qrun = items[1].x * 0.99
    items[2] = H.Item("w1", _rand(640, 303, 0.1), S, 1, synth.WEIGHT, 1)
    items[4].layer = 1
    res, out = run(items)
    rows = [H.check_item(t, it, res) for t, it in enumerate(items[:4])]
    o_order, _ = orc.rank_layers([rows[0]["w_sqnr"], rows[2]["w_sqnr"]], [rows[1]["p_sqnr"], rows[3]["p_sqnr"]],
                                 [rows[0]["w_mse"], rows[2]["w_mse"]], [rows[1]["p_mse"], rows[3]["p_mse"]])
    assert out.order[:2].tolist() == o_order and np.isfinite(out.score[:2]).all()
    assert np.isnan(out.metrics["mse"][4])
    # (2) a NaN inside a ranked activation: layer order, NaN scores
    items = _poisoned_set()[:4]
    res, out = run(items)
    assert out.order[:2].tolist() == [0, 1] and np.isnan(out.score[:2]).all()


def test_two_plans_on_two_streams_at_once():
    """Different plans are independent: two of them, each with its own workspace and outputs, run
    at the same time on two streams, several passes each, and reproduce their serial results bit
    for bit (parameters, sums, pair sums, codes)."""
    sets = [synth.config_resnet18(4), synth.config_mobilenetv2(4)]
    jobs = []
    for specs in sets:
        items = H.items_from_specs(specs, DEV)
        for it in items:
            if it.kind == synth.ACTIVATION:
                it.qrun = it.x * 0.97 + 0.002
        res = H.run_gpu(items, fused="single")                     # serial reference
        want = [res.buffers.params.clone(), res.buffers.sums.clone(), res.buffers.pair.clone()] + \
               [it.codes.clone() for it in items]
        jobs.append((items, res, want, qb.Buffers(res.plan, DEV), torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(3):
        for items, res, want, buf, st in jobs:
            for it in items:
                it.codes.fill_(0x11)
            for b in (buf.params, buf.sums, buf.pair, buf.workspace):
                b.fill_(0x5A)
        torch.cuda.synchronize()
        for k in range(4):                                         # interleaved: both streams stay busy
            for items, res, want, buf, st in jobs:
                qb.qv2_calibrate_fakequant_pair_metrics(res.plan, buf.params, buf.sums, buf.pair, buf.workspace,
                                                        stream=st)
        torch.cuda.synchronize()
        for j, (items, res, want, buf, st) in enumerate(jobs):
            got = [buf.params, buf.sums, buf.pair] + [it.codes for it in items]
            assert all(torch.equal(a, b) for a, b in zip(got, want)), f"plan {j}, round {rep}"


@pytest.mark.parametrize("fused", [False, True, "single"])
def test_large_pair_at_different_offsets_inside_16_bytes(fused):
    """x and its partner start at different offsets inside 16 bytes (every combination), long
    enough for many tiles: the partner is read as vectors from 4-byte aligned addresses."""
    n = 1_000_003
    items = []
    for ox in range(4):
        for oq in range(4):
            if ox == oq:
                continue
            x = torch.relu(_rand(n + 8, 700 + ox)[ox: ox + n])
            q = _rand(n + 8, 710 + 4 * ox + oq)[oq: oq + n] * 0.01 + x
            items.append(H.Item(f"x+{ox}.q+{oq}", x, A, 1, synth.ACTIVATION, len(items), qrun=q,
                                codes_offset=(ox + oq) % 4))
    res = H.run_gpu(items, fused=fused)
    H.check_all(items, res)


def test_pass_records_equal_single_call_plus_tensor_fold():
    """qv2_sensitivity_pass makes its per-tensor records inside its last fold launch (single-segment
    tensors with their segment, row-group tensors by one more workgroup each, tensors of several
    stream segments by a small launch after it); they must be, bit for bit, what the single call
    followed by qv2_tensor_sums_fold gives, and so must parameters, sums and codes."""
    specs = synth.config_mobilenetv2(2)
    items = H.items_from_specs(specs, DEV)
    for it in items:
        if it.kind == synth.ACTIVATION:
            it.qrun = it.x * 0.98 + 0.003
    n0 = len(items)
    # rows held by 512-thread workgroups, rows cut into stream tiles (odd length: several segments
    # per tensor), a one-channel row tensor, a weight with a partner in the row kernels
    extra = [H.Item("wide", _rand(5 * 25088, 901, 0.1), C, 5, synth.WEIGHT, 0),
             H.Item("late", _rand(3 * 20001, 902, 0.1), C, 3, synth.WEIGHT, 0),
             H.Item("one-row", _rand(576, 903, 0.1), C, 1, synth.WEIGHT, 0),
             H.Item("row+pair", _rand(64 * 576, 904, 0.1), C, 64, synth.WEIGHT, 0)]
    extra[3].qrun = extra[3].x * 1.01
    n_layers = max(it.layer for it in items[:n0]) + 2
    for it in extra[:3]:
        it.kind, it.layer = 2, 0                   # neither weight nor activation: not ranked
    extra[3].layer = n_layers - 1                  # one more layer: this weight and an activation
    act = H.Item("extra.out", torch.relu(_rand(40_000, 905)), A, 1, synth.ACTIVATION, n_layers - 1)
    act.qrun = act.x * 0.99
    items += extra + [act]
    res = H.run_gpu(items, fused="single")
    want_codes = [it.codes.clone() for it in items]
    buf = qb.Buffers(res.plan, DEV)
    out = qb.PassOutputs(res.plan, n_layers, DEV)
    for it in items:
        it.codes.fill_(0x33)
    qb.qv2_sensitivity_pass(res.plan, buf.params, buf.sums, out, buf.workspace)
    p, s, _ = buf.host()
    assert p.tobytes() == res.params.tobytes() and s.tobytes() == res.sums.tobytes()
    assert out.tensor_sums.tobytes() == res.tsums.tobytes()
    assert out.pair_sums.tobytes() == res.pair.tobytes()
    assert all(torch.equal(it.codes, w) for it, w in zip(items, want_codes))
    # h_records in ordinary (pageable) host memory: the records come over by a copy instead of being
    # written there by the folds; same bytes
    import ctypes
    nt = res.plan.num_tensors
    h_plain = np.zeros(nt * (qb.TENSOR_SUMS.itemsize + qb.PAIR_SUMS.itemsize), np.uint8)
    order = np.zeros(n_layers, np.int32)
    st = qb.lib().qv2_sensitivity_pass(res.plan.handle, buf.params.data_ptr(), buf.sums.data_ptr(),
                                       out.d_records.data_ptr(), h_plain.ctypes.data, buf.workspace.data_ptr(),
                                       buf.workspace.numel(), None, None, n_layers, None, None, None, None,
                                       order.ctypes.data, None)
    assert st == qb.QV2_OK and order.tolist() == out.order.tolist()
    assert h_plain.tobytes() == out.h_records.numpy().tobytes()
    assert out.d_records.cpu().numpy().tobytes() == h_plain.tobytes()       # the device copy is written too
    # and the two halves of the pass give the same again
    prep = qb.PreparedPass(res.plan, buf.params, buf.sums, [out, qb.PassOutputs(res.plan, n_layers, DEV)],
                           buf.workspace)
    prep.begin(1)
    o1 = prep.end(1)
    assert o1.tensor_sums.tobytes() == res.tsums.tobytes() and o1.order.tolist() == out.order.tolist()
