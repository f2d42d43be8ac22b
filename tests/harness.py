"""Shared plumbing of the GPU parity tests: feed the same bytes to the HIP
library (through the ctypes binding of the C ABI) and to the CPU oracle, and
compare to the stated bar.

Bar (from the benchmark spec): min, max, scale, zero-point and int8 codes
bit-exact; MSE within 1e-4 relative; SQNR within 1e-3 dB; ranking identical.
Added here: sum(x^2) within 1e-6 relative, mean within 1e-6 * absmax, variance
within 1e-4 relative.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from oracle import reference as orc
from paper_2501_07161_amd import binding as qb
from paper_2501_07161_amd import synth

MSE_RTOL = 1e-4
SQNR_ATOL_DB = 1e-3
SX2_RTOL = 1e-6
VAR_RTOL = 1e-4
COS_ATOL = 1e-9        # cosine similarity: fp64 sums, norms recovered from energy differences


@dataclass
class Item:
    """One tensor of a case: device data plus how to quantize it."""
    name: str
    x: torch.Tensor                      # device, fp32 (any view with a valid data_ptr)
    scheme: int = qb.QV2_ASYM_TENSOR
    channels: int = 1
    kind: int = 0
    layer: int = 0
    qrun: Optional[torch.Tensor] = None
    want_codes: bool = True
    codes: Optional[torch.Tensor] = None  # filled by run_gpu
    codes_offset: int = 0                 # byte misalignment to give the code buffer (tests)


@dataclass
class GpuResult:
    plan: qb.Plan
    params: np.ndarray
    sums: np.ndarray
    pair: np.ndarray
    metrics: np.ndarray
    pair_mse: np.ndarray
    pair_sqnr: np.ndarray


def workers() -> int:
    return max(1, min(8, (os.cpu_count() or 1)))


def items_from_specs(specs: List[synth.TensorSpec], device="cuda") -> List[Item]:
    out = []
    for s in specs:
        x = synth.materialize(s, device)
        out.append(Item(s.name, x, s.scheme, s.channels, s.kind, s.layer))
    return out


def attach_pairs(items: List[Item], specs: List[synth.TensorSpec]):
    """Quantized-run partner of every activation: dequant(quant(ref)) + N(0, (0.01*std(ref))^2),
    made by the ORACLE from the host copy of ref (never by the HIP path)."""
    def one(idx):
        it, sp = items[idx], specs[idx]
        if not sp.has_pair:
            return None
        x = it.x.detach().cpu().numpy().reshape(-1)
        cal = orc.calibrate(x, it.scheme, it.channels)
        fq = orc.fakequant(x, cal, it.scheme, it.channels, keep_xhat=True)
        noise = synth.unit_noise(sp, it.x.device).cpu().numpy().reshape(-1)
        sigma = np.float32(0.01 * float(np.std(x, dtype=np.float64)))
        noise *= sigma
        noise += fq.xhat
        fq.xhat = None
        it._oracle = (cal, fq)             # reused by check_item: same oracle, same input bytes
        return noise
    with ThreadPoolExecutor(workers()) as ex:
        res = list(ex.map(one, range(len(items))))
    for it, q in zip(items, res):
        if q is not None:
            it.qrun = torch.from_numpy(q).to(it.x.device).view(it.x.shape)


def run_gpu(items: List[Item], params_override: Optional[np.ndarray] = None,
            do_calibrate: bool = True, fused: bool = False, cos: bool = False) -> GpuResult:
    """calibrate -> fakequant -> pair (fused=True: the fused fakequant+pair call;
    fused="single": the one call that does all three) on the current stream, then host
    finalize."""
    dev = items[0].x.device
    rows = []
    for it in items:
        if it.want_codes:
            raw = torch.full((it.x.numel() + 16,), 0x55, dtype=torch.int8, device=dev)
            it._raw_codes = raw
            it.codes = raw[it.codes_offset: it.codes_offset + it.x.numel()]
        rows.append(qb.TensorArg(x=it.x, numel=it.x.numel(), scheme=it.scheme, channels=it.channels,
                                 qrun=it.qrun, codes=it.codes if it.want_codes else None,
                                 kind=it.kind, layer=it.layer))
    plan = qb.qv2_plan_create(rows)
    buf = qb.Buffers(plan, dev)
    single = fused == "single"
    assert not (single and (params_override is not None or not do_calibrate))
    if do_calibrate and not single:
        qb.qv2_calibrate(plan, buf.params, buf.sums, buf.workspace)
    if params_override is not None:
        torch.cuda.synchronize()
        buf.params.copy_(torch.from_numpy(params_override.view(np.uint8)).to(dev))
    seg_xxhat = pair_xq = None
    if cos:
        seg_xxhat = torch.zeros(plan.num_segments, dtype=torch.float64, device=dev)
        pair_xq = torch.zeros(plan.num_tensors, dtype=torch.float64, device=dev)
        if single:
            qb.qv2_calibrate_fakequant_pair_metrics_cos(plan, buf.params, buf.sums, buf.pair, seg_xxhat,
                                                        pair_xq, buf.workspace)
        else:
            qb.qv2_fakequant_pair_metrics_cos(plan, buf.params, buf.sums, buf.pair, seg_xxhat, pair_xq,
                                              buf.workspace)
    elif single:
        qb.qv2_calibrate_fakequant_pair_metrics(plan, buf.params, buf.sums, buf.pair, buf.workspace)
    elif fused:
        qb.qv2_fakequant_pair_metrics(plan, buf.params, buf.sums, buf.pair, buf.workspace)
    else:
        qb.qv2_fakequant_metrics(plan, buf.params, buf.sums, buf.workspace)
        qb.qv2_pair_metrics(plan, buf.pair, buf.workspace)
    tsums = torch.zeros(plan.num_tensors * qb.TENSOR_SUMS.itemsize, dtype=torch.uint8, device=dev)
    qb.qv2_tensor_sums_fold(plan, buf.params, buf.sums, tsums)
    torch.cuda.synchronize()
    params, sums, pair = buf.host()
    metrics = qb.qv2_finalize(plan, params, sums, strict=False)
    # the device-side per-tensor fold gives the same metrics (channel sums in another order)
    m2 = qb.qv2_finalize_tensors(tsums.cpu().numpy().view(qb.TENSOR_SUMS), strict=False)
    for f, rt in (("mse", 1e-12), ("mean", 1e-9), ("var", 1e-8)):
        assert np.allclose(m2[f], metrics[f], rtol=rt, atol=1e-300, equal_nan=True), f
    with np.errstate(invalid="ignore"):
        same = (m2["sqnr_db"] == metrics["sqnr_db"]) | (np.abs(m2["sqnr_db"] - metrics["sqnr_db"]) <= 1e-9) | \
               (np.isnan(m2["sqnr_db"]) & np.isnan(metrics["sqnr_db"]))
    assert np.all(same)
    for f in ("min", "max", "absmax"):
        assert np.array_equal(m2[f], metrics[f], equal_nan=True), f
    pm, ps = qb.qv2_pair_finalize(pair, strict=False)
    res = GpuResult(plan, params, sums, pair, metrics, pm, ps)
    res.buffers = buf
    res.tsums = tsums.cpu().numpy().view(qb.TENSOR_SUMS)
    res.cos_quant = res.cos_pair = None
    if cos:
        res.cos_quant, res.cos_pair = qb.qv2_cosine_finalize(plan, sums, seg_xxhat.cpu().numpy(), pair,
                                                             pair_xq.cpu().numpy(), strict=False)
    return res


def _rel(a, b):
    return abs(a - b) / max(abs(b), 1e-300)


def check_item(t: int, it: Item, res: GpuResult, check_codes: bool = True, cal=None):
    """Element-by-element comparison of one tensor against the oracle."""
    x = it.x.detach().cpu().numpy().reshape(-1)
    if cal is None and getattr(it, "_oracle", None) is not None:
        cal, fq = it._oracle
    else:
        cal = cal or orc.calibrate(x, it.scheme, it.channels)
        fq = orc.fakequant(x, cal, it.scheme, it.channels)
    s0 = res.plan.segment_begin[t]
    S = it.channels if it.scheme == qb.QV2_SYM_CHANNEL else 1
    P, U = res.params[s0:s0 + S], res.sums[s0:s0 + S]
    tag = f"{it.name} (tensor {t})"
    # bit-exact part
    for fld, want in (("min", cal.min), ("max", cal.max), ("scale", cal.scale),
                      ("inv_scale", cal.inv_scale)):
        got = P[fld]
        bad = np.nonzero(got.view(np.uint32) != want.view(np.uint32))[0]
        assert bad.size == 0, f"{tag}: {fld} differs at segment {bad[:5]}: {got[bad[:5]]} vs {want[bad[:5]]}"
    assert np.array_equal(P["zp"], cal.zp), f"{tag}: zero-point"
    assert np.array_equal(U["n"], cal.n), f"{tag}: n"
    if check_codes and it.want_codes:
        got = it.codes.cpu().numpy()
        bad = np.nonzero(got != fq.codes)[0]
        assert bad.size == 0, (f"{tag}: {bad.size} codes differ, first at {bad[:5]}: "
                               f"{got[bad[:5]]} vs {fq.codes[bad[:5]]}")
        raw = it._raw_codes.cpu().numpy()     # nothing written outside the code range
        assert np.all(raw[:it.codes_offset] == 0x55) and np.all(raw[it.codes_offset + x.size:] == 0x55), \
            f"{tag}: code buffer overrun"
    # floating-point part, per segment
    absmax = np.maximum(np.abs(cal.min), np.abs(cal.max)).astype(np.float64)
    n = cal.n.astype(np.float64)
    assert np.all(np.abs(U["sum_x"] - cal.sum_x) / n <= 1e-6 * absmax + 1e-300), f"{tag}: sum_x"
    assert np.all(np.abs(U["sum_x2"] - fq.sum_x2) <= SX2_RTOL * fq.sum_x2 + 1e-300), f"{tag}: sum_x2"
    assert np.all(np.abs(U["sum_e2"] - fq.sum_e2) <= MSE_RTOL * fq.sum_e2 + 1e-300), f"{tag}: sum_e2"
    # per tensor
    m = orc.tensor_metrics(x, cal, fq)
    g = res.metrics[t]
    assert _rel(g["mse"], m.mse) <= MSE_RTOL or (m.mse == 0 and g["mse"] == 0), f"{tag}: mse {g['mse']} vs {m.mse}"
    if math.isinf(m.sqnr_db):
        assert g["sqnr_db"] == m.sqnr_db, f"{tag}: sqnr"
    else:
        assert abs(g["sqnr_db"] - m.sqnr_db) <= SQNR_ATOL_DB, f"{tag}: sqnr {g['sqnr_db']} vs {m.sqnr_db}"
    assert abs(g["mean"] - m.mean) <= 1e-6 * m.absmax + 1e-300, f"{tag}: mean"
    assert abs(g["var"] - m.var) <= VAR_RTOL * m.var + 1e-12, f"{tag}: var {g['var']} vs {m.var}"
    assert g["absmax"] == np.float32(m.absmax) and g["min"] == np.float32(m.min) and g["max"] == np.float32(m.max)
    out = {"w_mse": m.mse, "w_sqnr": m.sqnr_db}
    if getattr(res, "cos_quant", None) is not None:         # Eq. 8, tensor vs its dequantized form
        xhat = np.concatenate([orc.dequantize(fq.codes.reshape(S, -1)[c], cal.scale[c], cal.zp[c])
                               for c in range(S)])
        want = orc.cosine_similarity(x, xhat)
        assert abs(res.cos_quant[t] - want) <= COS_ATOL, f"{tag}: cos(x, xhat) {res.cos_quant[t]} vs {want}"
        if it.qrun is not None:
            want = orc.cosine_similarity(x, it.qrun.detach().cpu().numpy().reshape(-1))
            assert abs(res.cos_pair[t] - want) <= COS_ATOL, f"{tag}: cos(x, qrun) {res.cos_pair[t]} vs {want}"
        else:
            assert math.isnan(res.cos_pair[t])
    # pair
    if it.qrun is not None:
        pm = orc.pair_metrics(x, it.qrun.detach().cpu().numpy().reshape(-1))
        rec = res.pair[t]
        assert rec["n"] == x.size
        assert _rel(rec["sum_ref2"], pm.sum_ref2) <= SX2_RTOL, f"{tag}: pair sum_ref2"
        assert _rel(rec["sum_d2"], pm.sum_d2) <= MSE_RTOL or (pm.sum_d2 == 0 and rec["sum_d2"] == 0), \
            f"{tag}: pair sum_d2"
        assert _rel(res.pair_mse[t], pm.mse) <= MSE_RTOL or pm.mse == 0
        if math.isinf(pm.sqnr_db):
            assert res.pair_sqnr[t] == pm.sqnr_db
        else:
            assert abs(res.pair_sqnr[t] - pm.sqnr_db) <= SQNR_ATOL_DB, f"{tag}: pair sqnr"
        out.update(p_mse=pm.mse, p_sqnr=pm.sqnr_db)
    else:
        assert res.pair[t]["n"] == 0 and res.pair[t]["sum_d2"] == 0
    return out


def check_all(items: List[Item], res: GpuResult, parallel: bool = True):
    idx = range(len(items))
    if parallel and len(items) > 4:
        with ThreadPoolExecutor(workers()) as ex:
            return list(ex.map(lambda t: check_item(t, items[t], res), idx))
    return [check_item(t, items[t], res) for t in idx]


def check_ranking(items: List[Item], res: GpuResult, oracle_rows, cfg_kwargs=None):
    """Layer table -> per-layer series -> ranking, GPU metrics through qv2_rank
    against oracle metrics through the oracle's Algorithm 2.  Identical lists."""
    cfg_kwargs = cfg_kwargs or {}
    n_layers = max(it.layer for it in items) + 1
    g = {k: np.full(n_layers, np.nan) for k in ("w_sqnr", "a_sqnr", "w_mse", "a_mse")}
    o = {k: np.full(n_layers, np.nan) for k in ("w_sqnr", "a_sqnr", "w_mse", "a_mse")}
    for t, (it, row) in enumerate(zip(items, oracle_rows)):
        if it.kind == synth.WEIGHT:
            g["w_sqnr"][it.layer], g["w_mse"][it.layer] = res.metrics[t]["sqnr_db"], res.metrics[t]["mse"]
            o["w_sqnr"][it.layer], o["w_mse"][it.layer] = row["w_sqnr"], row["w_mse"]
        elif it.qrun is not None:
            g["a_sqnr"][it.layer], g["a_mse"][it.layer] = res.pair_sqnr[t], res.pair_mse[t]
            o["a_sqnr"][it.layer], o["a_mse"][it.layer] = row["p_sqnr"], row["p_mse"]
    if np.isnan(g["a_sqnr"]).any():        # a layer without an activation pair: weight series only
        cfg_kwargs = dict(cfg_kwargs, mse_source=1)
        for d in (g, o):
            d["a_sqnr"] = d["a_mse"] = None
    cfg = qb.qv2_rank_config_default()
    for k, v in cfg_kwargs.items():
        setattr(cfg, k, v)
    order, score = qb.qv2_rank(g["w_sqnr"], g["a_sqnr"], g["w_mse"], g["a_mse"], None, cfg)
    lst = lambda a: None if a is None else list(a)
    o_order, o_score = orc.rank_layers(lst(o["w_sqnr"]), lst(o["a_sqnr"]), lst(o["w_mse"]),
                                       lst(o["a_mse"]), None, orc.RankConfig(**cfg_kwargs))
    assert order.tolist() == o_order, f"ranking differs:\n gpu    {order.tolist()}\n oracle {o_order}"
    assert np.allclose(score, o_score, rtol=0, atol=2 * SQNR_ATOL_DB)
    if g["a_sqnr"] is not None and not np.isnan(g["w_sqnr"]).any():
        # every layer has a weight and an activation pair: the one-call form must agree
        order2, score2 = qb.qv2_rank_tensors(res.plan, res.tsums, res.pair, n_layers, None, cfg)
        assert order2.tolist() == o_order
        assert np.allclose(score2, o_score, rtol=0, atol=2 * SQNR_ATOL_DB)
        # ... and so must the whole pass as ONE native call, run again on the same plan
        buf = qb.Buffers(res.plan, items[0].x.device)
        out = qb.PassOutputs(res.plan, n_layers, items[0].x.device)
        order3, score3 = qb.qv2_sensitivity_pass(res.plan, buf.params, buf.sums, out, buf.workspace, cfg=cfg)
        assert order3.tolist() == o_order
        assert np.allclose(score3, o_score, rtol=0, atol=2 * SQNR_ATOL_DB)
        p3, s3, _ = buf.host()
        assert p3.tobytes() == res.params.tobytes()                        # same parameters, bit for bit
        assert np.array_equal(s3["sum_e2"], res.sums["sum_e2"]) and np.array_equal(s3["n"], res.sums["n"])
        assert np.allclose(out.metrics["mse"], res.metrics["mse"], rtol=1e-12, atol=0)
        assert np.allclose(out.pair_mse, res.pair_mse, rtol=1e-12, atol=0)
        assert np.array_equal(out.pair_sums["n"], res.pair["n"])
    return order.tolist()


def same_sums_single_call(single: np.ndarray, other: np.ndarray):
    """Per-segment sums of the single call against those of the separate calls: sum x, sum e^2 and
    n bit for bit; sum x^2 up to fp64 summation order for segments cut into stream tiles (the
    single call keeps the calibration sweep's sum instead of summing x^2 again while it
    quantizes), bit for bit for the others."""
    for f in ("sum_x", "sum_e2", "n"):
        assert np.array_equal(single[f], other[f], equal_nan=True), f
    assert np.allclose(single["sum_x2"], other["sum_x2"], rtol=1e-12, atol=0, equal_nan=True)
