"""Full-size parity in the launch configuration the benchmark times.  The MobileNetV2
batch-64 and VGG-16 batch-16 sets go through the single call and are compared element by
element.  The ResNet-50 v1
batch-256 set (54 per-channel weights, 54 activations of 10.8 GB with oracle-made
quantized-run partners) goes through ONE plan, as in bench.py, and every tensor is
compared with the CPU oracle: parameters and all 2.7 G int8 codes bit-exact, sums, MSE,
SQNR and the ranking to the stated bar; the fused call and the single call (the pass the
benchmark times) must then reproduce those records and codes.  The oracle runs on the host
cores in a thread pool (one tensor per call), which takes about a minute."""
import numpy as np
import pytest
import torch

import harness as H
from paper_2501_07161_amd import synth

pytestmark = pytest.mark.gpu


def test_resnet50_batch256_full_pass():
    specs = synth.config_resnet50(256)
    items = H.items_from_specs(specs, "cuda")
    print("oracle: calibrate + fake-quant + quantized-run partners ...", flush=True)
    H.attach_pairs(items, specs)
    print("gpu pass ...", flush=True)
    res = H.run_gpu(items)
    assert res.plan.num_tensors == 108
    print("compare ...", flush=True)
    rows = H.check_all(items, res)
    order = H.check_ranking(items, res, rows)
    assert sorted(order) == list(range(54))
    print("fused fake-quant + pair call ...", flush=True)
    codes = [it.codes for it in items]
    res2 = H.run_gpu(items, fused=True)            # fresh code buffers
    assert res2.params.tobytes() == res.params.tobytes()
    assert res2.sums.tobytes() == res.sums.tobytes()
    for f in ("sum_ref2", "sum_d2"):
        assert np.allclose(res2.pair[f], res.pair[f], rtol=1e-12, atol=0)
    assert all(torch.equal(a, it.codes) for a, it in zip(codes, items))
    print("single call (the pass bench.py times) ...", flush=True)
    del res, codes
    codes2 = [it.codes for it in items]
    res3 = H.run_gpu(items, fused="single")        # fresh code buffers
    assert res3.params.tobytes() == res2.params.tobytes()
    H.same_sums_single_call(res3.sums, res2.sums)
    for f in ("sum_ref2", "sum_d2"):
        assert np.allclose(res3.pair[f], res2.pair[f], rtol=1e-12, atol=0)
    assert np.array_equal(res3.pair["n"], res2.pair["n"])
    assert all(torch.equal(a, it.codes) for a, it in zip(codes2, items))
    # the fused-IR variant of the same set at the same batch (Sec. 6.3 Eq. 10-12: BN folded into
    # the weights): its 54 weights differ, its activations and partners are these very tensors.
    # One plan of 108 tensors through the single call again; the folded weights element by
    # element against the oracle, the activations against the records and codes just checked.
    print("BN-folded variant, single call ...", flush=True)
    fspecs = synth.config_resnet50(256, fused=True)
    fitems = []
    for it, sp in zip(items, fspecs):
        assert sp.name == it.name
        if sp.kind == synth.WEIGHT:
            fitems.append(H.Item(sp.name, synth.materialize(sp, "cuda"), sp.scheme, sp.channels, sp.kind, sp.layer))
        else:
            fitems.append(it)
    res4 = H.run_gpu(fitems, fused="single")       # fresh code buffers for every tensor
    w_idx = [t for t, sp in enumerate(fspecs) if sp.kind == synth.WEIGHT]
    a_idx = [t for t, sp in enumerate(fspecs) if sp.kind == synth.ACTIVATION]
    assert any(not torch.equal(fitems[t].x, synth.materialize(specs[t], "cuda")) for t in w_idx[:3])
    for t in w_idx:
        H.check_item(t, fitems[t], res4)
    for t in a_idx:
        s0 = res4.plan.segment_begin[t]
        assert res4.params[s0].tobytes() == res3.params[s0].tobytes()
        assert res4.sums[s0].tobytes() == res3.sums[s0].tobytes()
        assert res4.pair[t].tobytes() == res3.pair[t].tobytes()
        assert torch.equal(fitems[t].codes, codes2[t])
    del items, fitems
    torch.cuda.empty_cache()


def _full_set_single_call(specs, n_layers):
    """One plan over a whole set at its stated batch, through the single call (the pass the
    benchmark times), every element against the oracle."""
    items = H.items_from_specs(specs, "cuda")
    print("oracle: calibrate + fake-quant + quantized-run partners ...", flush=True)
    H.attach_pairs(items, specs)
    print("gpu pass (single call) ...", flush=True)
    res = H.run_gpu(items, fused="single")
    print("compare ...", flush=True)
    rows = H.check_all(items, res)
    order = H.check_ranking(items, res, rows)
    assert sorted(order) == list(range(n_layers))
    del items, res
    torch.cuda.empty_cache()


@pytest.mark.timeout(600)
def test_mobilenetv2_batch64_full_pass():
    """MobileNetV2 at batch 64: 53 per-channel weights (rows of 9 ... 1280 elements) and 53
    activations of 427 M elements with ReLU6 clipping, partners made by the oracle."""
    _full_set_single_call(synth.config_mobilenetv2(64), 53)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("per_channel", [False, True])
def test_vgg16_batch16_full_pass(per_channel):
    """VGG-16 at batch 16: 138 M weight elements (fc6 alone 411 MB; per-channel rows of up to
    25088 elements) and 217 M activation elements."""
    _full_set_single_call(synth.config_vgg16(16, per_channel), 16)


@pytest.mark.timeout(900)
def test_single_tensor_beyond_int32_elements():
    """One activation of 2^31 + 4099 elements (8.6 GB) with its quantized-run partner: element
    offsets, tile counts and segment lengths no longer fit 32 bits.  All codes bit-exact."""
    n = (1 << 31) + 4099
    spec = synth.TensorSpec("huge_act", (n,), synth.ACTIVATION, 0, synth.ASYM_TENSOR, 9001, "relu_normal",
                            sigma=1.3, has_pair=True)
    items = H.items_from_specs([spec], "cuda")
    print("oracle: calibrate + fake-quant + partner ...", flush=True)
    H.attach_pairs(items, [spec])
    for fused in (False, True):
        print(f"gpu pass (fused={fused}) ...", flush=True)
        res = H.run_gpu(items, fused=fused)
        assert int(res.sums["n"][0]) == n
        print("compare ...", flush=True)
        H.check_item(0, items[0], res)
    del items
    torch.cuda.empty_cache()
