"""The entry point that allocates nothing (qv2_calibrate_fakequant_pair_metrics_noalloc, for
callers that cannot call hipMalloc) against the entry point with a workspace argument, through
the C ABI: two calls in a row on the library's fixed device array, the second on a smaller
input, so whatever the first call left there must not matter."""
import numpy as np
import pytest
import torch

from paper_2501_07161_amd import binding as qb
from paper_2501_07161_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _rows(specs):
    xs = [synth.materialize(s, DEV) for s in specs]
    rows, keep = [], []
    for s, x in zip(specs, xs):
        q = None
        if s.has_pair:      # any partner will do here: both entry points read the same bytes
            q = x * 0.98 + 0.003 * synth.unit_noise(s, DEV)
        c = torch.full((x.numel(),), 0x55, dtype=torch.int8, device=DEV)
        rows.append(qb.TensorArg(x=x, numel=x.numel(), scheme=s.scheme, channels=s.channels, qrun=q,
                                 codes=c, kind=s.kind, layer=s.layer))
        keep.append(c)
    return rows, keep


def _both_ways(specs):
    rows, codes = _rows(specs)
    plan = qb.qv2_plan_create(rows)
    assert plan.workspace_bytes <= qb.QV2_STATIC_SCRATCH_BYTES
    # reference: the existing entry point, workspace from the caller
    ref = qb.Buffers(plan, DEV)
    qb.qv2_calibrate_fakequant_pair_metrics(plan, ref.params, ref.sums, ref.pair, ref.workspace)
    torch.cuda.synchronize()
    want = [b.copy() for b in ref.host()]
    want_codes = [c.cpu().numpy().copy() for c in codes]
    for c in codes:
        c.fill_(0x55)
    # the entry point under test: output buffers only; they exist before the call, and the
    # call itself is bracketed by a check that torch's allocator was not asked for anything
    out = qb.Buffers(plan, DEV)
    del out.workspace
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    qb.qv2_calibrate_fakequant_pair_metrics_noalloc(plan, out.params, out.sums, out.pair)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before
    got = (out.params.cpu().numpy().view(qb.QPARAMS), out.sums.cpu().numpy().view(qb.SUMS),
           out.pair.cpu().numpy().view(qb.PAIR_SUMS))
    # same kernels, same fold order: parameters, codes (bit-exact bar) and every sum (1e-4 / 1e-6
    # relative bar) agree bit for bit
    for g, w, name in zip(got, want, ("params", "sums", "pair")):
        assert g.tobytes() == w.tobytes(), name
    for t, (c, w) in enumerate(zip(codes, want_codes)):
        assert np.array_equal(c.cpu().numpy(), w), f"codes of tensor {t}"
    assert np.all(np.isfinite(got[1]["sum_e2"])) and np.all(got[1]["n"] > 0)
    plan.close()


def test_no_alloc_entry_point_matches_workspace_entry_point_twice():
    # first call: ResNet-50 shapes at batch 2 (per-channel weights in the row kernels, activations
    # with partners as stream tiles); second call: the three-tensor set, far smaller
    _both_ways(synth.config_resnet50(2))
    _both_ways(synth.config_tiny())


def test_no_alloc_entry_point_refuses_what_it_cannot_serve():
    x = torch.randn(4096, device=DEV)
    plan = qb.qv2_plan_create([qb.TensorArg(x=x, numel=x.numel())])
    buf = qb.Buffers(plan, DEV)
    with pytest.raises(qb.QV2Error) as e:          # tables not on the device yet: it may not allocate
        qb.qv2_calibrate_fakequant_pair_metrics_noalloc(plan, buf.params, buf.sums, None)
    assert e.value.status == qb.QV2_ERR_STATE
    qb.qv2_plan_upload(plan)
    qb.qv2_calibrate_fakequant_pair_metrics_noalloc(plan, buf.params, buf.sums, None)
    torch.cuda.synchronize()
    p = buf.params.cpu().numpy().view(qb.QPARAMS)
    assert p["min"][0] == float(x.min()) and p["max"][0] == float(x.max())
    plan.close()
