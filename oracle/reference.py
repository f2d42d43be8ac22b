"""CPU oracle for the QuantuneV2 sensitivity pass -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``qv2_oracle.c`` (plain C, fp64 accumulation)
plus the host-side list logic of Sec. 6.4-6.5 (SQNR delta, Algorithm 2) written
as plain Python loops.  Nothing here is imported by the product package; only
the tests, the smoke check and the benchmark's ``cpu_baseline`` leg use it, and
it shares no code with the HIP library.

Per-segment conventions: a tensor is one segment (per-tensor schemes) or
``channels`` segments, one per slice along dim 0 (per-output-channel scheme;
the paper does not mention per-channel quantization -- Sec. 4 Eq. 4 is applied
to each output channel on its own, and a tensor's MSE / SQNR are formed from
the sums of its channels' sums).

Parity unpinned (the paper prints no value or rule to check against; the functions are pinned
to their stated readings only): the default gains alpha_w = 0.6 / alpha_a = 0.4 of
``rank_layers``, the smoothing constant ``eps`` of ``kl_divergence`` (no default), the histogram
binning rule of ``histogram``, the block-move rule of ``regroup_for_fusion``, and the text format
of ``config_text``.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

ASYM_TENSOR = 0   # Sec. 2.1 Eq. 1-3, whole tensor, range widened to hold 0
SYM_TENSOR = 1    # Sec. 4 Eq. 4-5, whole tensor
SYM_CHANNEL = 2   # Sec. 4 Eq. 4-5 per output channel (dim 0)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qv2_oracle.c")
_LIB = os.path.join(_HERE, "libqv2_oracle.so")
_lib = None

_F = ctypes.POINTER(ctypes.c_float)
_D = ctypes.POINTER(ctypes.c_double)
_I8 = ctypes.POINTER(ctypes.c_int8)
_I32 = ctypes.POINTER(ctypes.c_int32)
_I64 = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64 = ctypes.c_int64
        L.orc_minmax.argtypes = [_F, i64, _F, _F]
        L.orc_argminmax.argtypes = [_F, i64, _I64, _I64]
        L.orc_moments.argtypes = [_F, i64, _D, _D]
        L.orc_variance.argtypes = [_F, i64]
        L.orc_variance.restype = ctypes.c_double
        L.orc_params_asym.argtypes = [ctypes.c_float, ctypes.c_float, _F, _F, _I32]
        L.orc_params_sym.argtypes = [ctypes.c_float, ctypes.c_float, _F, _F, _I32]
        L.orc_quantize.argtypes = [_F, i64, ctypes.c_float, ctypes.c_int32, _I8]
        L.orc_dequantize.argtypes = [_I8, i64, ctypes.c_float, ctypes.c_int32, _F]
        L.orc_error_sums.argtypes = [_F, _F, i64, _D, _D]
        L.orc_histogram.argtypes = [_F, i64, ctypes.c_float, ctypes.c_float, ctypes.c_int32,
                                    ctypes.POINTER(ctypes.c_uint64)]
        L.orc_histogram.restype = None
        L.orc_bn_fold.argtypes = [_F, i64, i64, _F, _F, _F, _F, _F, _F, _F]
        L.orc_bn_fold.restype = None
        L.orc_cosine_sums.argtypes = [_F, _F, i64, _D, _D, _D]
        L.orc_cosine_sums.restype = None
        L.orc_mse.argtypes = [ctypes.c_double, i64]
        L.orc_mse.restype = ctypes.c_double
        L.orc_sqnr_db.argtypes = [ctypes.c_double, ctypes.c_double]
        L.orc_sqnr_db.restype = ctypes.c_double
        for name in ("orc_minmax", "orc_argminmax", "orc_moments", "orc_params_asym",
                     "orc_params_sym", "orc_quantize", "orc_dequantize", "orc_error_sums"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _f32(x) -> np.ndarray:
    a = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    return a


def _fp(a: np.ndarray):
    return a.ctypes.data_as(_F)


# ----------------------------------------------------------------------------
# element passes (each is one call into the C oracle)
# ----------------------------------------------------------------------------
def minmax(x):
    a = _f32(x)
    mn, mx = ctypes.c_float(), ctypes.c_float()
    lib().orc_minmax(_fp(a), a.size, ctypes.byref(mn), ctypes.byref(mx))
    return np.float32(mn.value), np.float32(mx.value)


def argminmax(x):
    a = _f32(x)
    i, j = ctypes.c_int64(), ctypes.c_int64()
    lib().orc_argminmax(_fp(a), a.size, ctypes.byref(i), ctypes.byref(j))
    return i.value, j.value


def moments(x):
    a = _f32(x)
    s, s2 = ctypes.c_double(), ctypes.c_double()
    lib().orc_moments(_fp(a), a.size, ctypes.byref(s), ctypes.byref(s2))
    return s.value, s2.value


def variance(x) -> float:
    a = _f32(x)
    return lib().orc_variance(_fp(a), a.size)


def params(mn, mx, scheme: int):
    """(scale, inv_scale, zp) for one segment from its min / max."""
    s, inv, zp = ctypes.c_float(), ctypes.c_float(), ctypes.c_int32()
    fn = lib().orc_params_asym if scheme == ASYM_TENSOR else lib().orc_params_sym
    if scheme not in (ASYM_TENSOR, SYM_TENSOR, SYM_CHANNEL):
        raise ValueError(f"unknown scheme {scheme}")
    fn(ctypes.c_float(float(mn)), ctypes.c_float(float(mx)),
       ctypes.byref(s), ctypes.byref(inv), ctypes.byref(zp))
    return np.float32(s.value), np.float32(inv.value), int(zp.value)


def quantize(x, inv_scale, zp) -> np.ndarray:
    a = _f32(x)
    q = np.empty(a.size, dtype=np.int8)
    lib().orc_quantize(_fp(a), a.size, ctypes.c_float(float(inv_scale)), int(zp),
                       q.ctypes.data_as(_I8))
    return q


def dequantize(q, scale, zp) -> np.ndarray:
    c = np.ascontiguousarray(q, dtype=np.int8).reshape(-1)
    out = np.empty(c.size, dtype=np.float32)
    lib().orc_dequantize(c.ctypes.data_as(_I8), c.size, ctypes.c_float(float(scale)),
                         int(zp), _fp(out))
    return out


def error_sums(x, xhat):
    a, b = _f32(x), _f32(xhat)
    if a.size != b.size:
        raise ValueError("size mismatch")
    s2, e2 = ctypes.c_double(), ctypes.c_double()
    lib().orc_error_sums(_fp(a), _fp(b), a.size, ctypes.byref(s2), ctypes.byref(e2))
    return s2.value, e2.value


def cosine_similarity(a, b) -> float:
    """Sec. 6.1 Eq. 8: A.B / (|A| |B|), fp64.  The paper does not say what a zero vector
    gives; reading taken: two zero vectors are identical (1), one zero vector gives 0."""
    x, y = _f32(a), _f32(b)
    if x.size != y.size:
        raise ValueError("size mismatch")
    sab, saa, sbb = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    lib().orc_cosine_sums(_fp(x), _fp(y), x.size, ctypes.byref(sab), ctypes.byref(saa), ctypes.byref(sbb))
    if saa.value == 0.0 or sbb.value == 0.0:
        return 1.0 if saa.value == sbb.value else 0.0
    return sab.value / (math.sqrt(saa.value) * math.sqrt(sbb.value))


def mse(sum_e2: float, n: int) -> float:
    return lib().orc_mse(sum_e2, n)


def sqnr_db(sum_x2: float, sum_e2: float) -> float:
    return lib().orc_sqnr_db(sum_x2, sum_e2)


# ----------------------------------------------------------------------------
# per-tensor composition: steps 1-3 of the paper's execution process (Sec. 4)
# ----------------------------------------------------------------------------
@dataclass
class Calibration:
    """Per-segment calibration of one tensor (arrays of length n_segments)."""
    min: np.ndarray
    max: np.ndarray
    scale: np.ndarray
    inv_scale: np.ndarray
    zp: np.ndarray
    sum_x: np.ndarray
    sum_x2: np.ndarray
    n: np.ndarray


@dataclass
class FakeQuant:
    codes: np.ndarray            # int8, flat, same element order as the tensor
    sum_x2: np.ndarray           # per segment
    sum_e2: np.ndarray           # per segment
    xhat: np.ndarray | None = None


@dataclass
class TensorMetrics:
    mse: float
    sqnr_db: float
    mean: float
    var: float
    absmax: float
    min: float
    max: float


def _segments(x, scheme: int, channels: int):
    a = _f32(x)
    if scheme == SYM_CHANNEL:
        if channels <= 0 or a.size % channels:
            raise ValueError("channels must divide numel")
        return a.reshape(channels, a.size // channels)
    if scheme in (ASYM_TENSOR, SYM_TENSOR):
        return a.reshape(1, a.size)
    raise ValueError(f"unknown scheme {scheme}")


def calibrate(x, scheme: int = ASYM_TENSOR, channels: int = 1) -> Calibration:
    seg = _segments(x, scheme, channels)
    S = seg.shape[0]
    out = Calibration(np.empty(S, np.float32), np.empty(S, np.float32), np.empty(S, np.float32),
                      np.empty(S, np.float32), np.empty(S, np.int32), np.empty(S, np.float64),
                      np.empty(S, np.float64), np.full(S, seg.shape[1], np.int64))
    for c in range(S):
        mn, mx = minmax(seg[c])
        sc, inv, zp = params(mn, mx, scheme)
        sx, sx2 = moments(seg[c])
        out.min[c], out.max[c], out.scale[c], out.inv_scale[c], out.zp[c] = mn, mx, sc, inv, zp
        out.sum_x[c], out.sum_x2[c] = sx, sx2
    return out


def fakequant(x, cal: Calibration, scheme: int = ASYM_TENSOR, channels: int = 1,
              keep_xhat: bool = False) -> FakeQuant:
    seg = _segments(x, scheme, channels)
    S, inner = seg.shape
    codes = np.empty((S, inner), np.int8)
    xhat_all = np.empty((S, inner), np.float32) if keep_xhat else None
    sx2 = np.empty(S, np.float64)
    se2 = np.empty(S, np.float64)
    for c in range(S):
        q = quantize(seg[c], cal.inv_scale[c], cal.zp[c])
        xh = dequantize(q, cal.scale[c], cal.zp[c])
        sx2[c], se2[c] = error_sums(seg[c], xh)
        codes[c] = q
        if keep_xhat:
            xhat_all[c] = xh
    return FakeQuant(codes.reshape(-1), sx2, se2,
                     xhat_all.reshape(-1) if keep_xhat else None)


def tensor_metrics(x, cal: Calibration, fq: FakeQuant) -> TensorMetrics:
    """Sec. 6.1 Eq. 6-7 plus the tensor statistics, one value per tensor."""
    a = _f32(x)
    n = a.size
    e2 = math.fsum(fq.sum_e2.tolist())
    x2 = math.fsum(fq.sum_x2.tolist())
    mn = float(np.min(cal.min))
    mx = float(np.max(cal.max))
    return TensorMetrics(mse=mse(e2, n), sqnr_db=sqnr_db(x2, e2),
                         mean=math.fsum(cal.sum_x.tolist()) / n, var=variance(a),
                         absmax=max(abs(mn), abs(mx)), min=mn, max=mx)


@dataclass
class PairMetrics:
    sum_ref2: float
    sum_d2: float
    n: int
    mse: float = field(init=False)
    sqnr_db: float = field(init=False)

    def __post_init__(self):
        self.mse = mse(self.sum_d2, self.n)
        self.sqnr_db = sqnr_db(self.sum_ref2, self.sum_d2)


def pair_metrics(ref, qrun) -> PairMetrics:
    """Algorithm 2's CalculateSQNR / CalculateMSE on a layer's output from the
    fp32 inference (D[i]) and from the quantized inference (Q[i])."""
    s2, d2 = error_sums(ref, qrun)
    return PairMetrics(s2, d2, int(np.asarray(ref).size))


# ----------------------------------------------------------------------------
# Sec. 6.4 Eq. 16 and Algorithm 2 (host-side list logic, plain Python)
# ----------------------------------------------------------------------------
@dataclass
class RankConfig:
    alpha_w: float = 0.6       # gain of the weight SQNR delta (larger than the activation's; the value is not printed)
    alpha_a: float = 0.4       # gain of the activation SQNR delta
    mse_factor: float = 5.0    # Algorithm 2: MSE above 5x the mean is an outlier
    mse_source: int = 0        # 0 activation-pair MSE, 1 weight MSE, 2 either (each vs its own mean)
    sqnr_cap_db: float = 200.0  # |SQNR| is clamped to this before differencing (no inf - inf)


def sqnr_deltas(sqnr, pos=None, cap_db: float = 200.0):
    """Eq. 16: delta_n = (SQNR_n - SQNR_{n-1}) / (L_n - L_{n-1}); delta_0 = 0."""
    n = len(sqnr)
    if pos is None:
        pos = list(range(n))
    s = []
    for v in sqnr:
        v = float(v)
        if math.isnan(v):
            raise ValueError("NaN SQNR")
        s.append(max(-cap_db, min(cap_db, v)))
    out = [0.0] * n
    for i in range(1, n):
        dl = pos[i] - pos[i - 1]
        if dl <= 0:
            raise ValueError("layer positions must increase")
        out[i] = (s[i] - s[i - 1]) / dl
    return out


def rank_layers(w_sqnr, a_sqnr, w_mse, a_mse, pos=None, cfg: RankConfig | None = None):
    """Algorithm 2 with RankLayersBySensitivity.  Returns (order, score): order[0]
    is the layer to keep in fp32 first."""
    cfg = cfg or RankConfig()
    n = len(w_sqnr) if w_sqnr is not None else len(a_sqnr)
    dw = sqnr_deltas(w_sqnr, pos, cfg.sqnr_cap_db) if w_sqnr is not None else [0.0] * n
    da = sqnr_deltas(a_sqnr, pos, cfg.sqnr_cap_db) if a_sqnr is not None else [0.0] * n
    G = [cfg.alpha_w * dw[i] + cfg.alpha_a * da[i] for i in range(n)]

    sources = {0: [a_mse], 1: [w_mse], 2: [w_mse, a_mse]}[cfg.mse_source]
    key = [0.0] * n             # ordering key of the outliers
    is_out = [False] * n
    for M in sources:
        if M is None:
            raise ValueError("MSE list required by mse_source is missing")
        M = [float(m) for m in M]
        if any(math.isnan(m) or math.isinf(m) or m < 0 for m in M):
            raise ValueError("non-finite MSE")
        total = 0.0
        for m in M:                 # the mean MSE of Algorithm 2: plain running sum over the layers
            total += m
        mean = total / n if n else 0.0
        for i in range(n):
            if M[i] > cfg.mse_factor * mean:
                is_out[i] = True
            k = M[i] if len(sources) == 1 else (M[i] / mean if mean > 0 else 0.0)
            key[i] = max(key[i], k)

    # Algorithm 2 ends with two groups.  The MSE outliers lead, the largest first (equal ones in
    # layer order); every other layer follows by score, the largest SQNR drop (most negative
    # score) first, equal scores in layer order.
    head = sorted((i for i in range(n) if is_out[i]), key=lambda i: (-key[i], i))
    rest = sorted((i for i in range(n) if not is_out[i]), key=lambda i: (G[i], i))
    return head + rest, G


# ----------------------------------------------------------------------------
# Sec. 7: baseline orders and the BOPs reduction rate (Eq. 17), plain Python
# ----------------------------------------------------------------------------
INORDER = 0
WEIGHT_SQNR_ORDER = 1


def baseline_order(kind: int, w_sqnr=None, n: int | None = None):
    """Sensitivity lists of the two compile-time baselines, in this library's convention
    (index 0 = the layer kept in fp32 first).
    InOrder quantizes from the first layer on, so the layers still in fp32 at any budget are
    the last ones: n-1, n-2, ..., 0.  Weight SQNR Order lists layers by ascending weight SQNR
    (equal values keep layer order)."""
    if kind == INORDER:
        n = len(w_sqnr) if n is None else n
        return list(range(n - 1, -1, -1))
    if kind == WEIGHT_SQNR_ORDER:
        vals = [float(v) for v in w_sqnr]
        if any(math.isnan(v) for v in vals):
            raise ValueError("NaN SQNR")
        return sorted(range(len(vals)), key=lambda i: (vals[i], i))
    raise ValueError(f"unknown baseline {kind}")


def bops_reduction_pct(macs, keep_fp32) -> float:
    """Eq. 17: (1 - BOPs(theta) / BOPs_fp32) * 100 with bits(theta_i) in {8, 32}."""
    total = 0.0
    mixed = 0.0
    for m, k in zip(macs, keep_fp32):
        total += 32.0 * float(m)
        mixed += (32.0 if k else 8.0) * float(m)
    return (1.0 - mixed / total) * 100.0


def bops_select(order, macs, target_pct: float):
    """Walk the sensitivity list from its head and keep layers in fp32 while the BOPs
    reduction rate stays at or above target_pct; stop at the first layer that would push it
    below.  Returns (keep_fp32 flags by layer, number kept, achieved rate)."""
    n = len(macs)
    if sorted(order) != list(range(n)):
        raise ValueError("order is not a permutation")
    if any((not math.isfinite(float(m))) or float(m) < 0 for m in macs) or not any(float(m) > 0 for m in macs):
        raise ValueError("bad MAC counts")
    keep = [False] * n
    kept = 0
    for l in order:
        keep[l] = True
        if bops_reduction_pct(macs, keep) < target_pct:
            keep[l] = False
            break
        kept += 1
    return keep, kept, bops_reduction_pct(macs, keep)


def config_text(keep_fp32, names=None) -> str:
    """Sec. 4 step 5: the configuration that states the bit-width of every layer - 32 for the
    layers kept in fp32, 8 for the rest.  The paper hands it to its compiler and prints no
    format; the one taken here is a text table, one line per layer in layer order:
    a header line ``layer,name,bits`` and then ``<index>,<name>,<32|8>`` (name = ``layer<index>``
    when none is given).  Parity of the format with the paper is unpinned."""
    lines = ["layer,name,bits"]
    for i, k in enumerate(keep_fp32):
        name = names[i] if names is not None else f"layer{i}"
        if any(c in name for c in ",\n\r"):
            raise ValueError("a layer name holds a comma or a line break")
        lines.append(f"{i},{name},{32 if k else 8}")
    return "\n".join(lines) + "\n"


# ----------------------------------------------------------------------------
# Sec. 5 calibration histograms and the KL divergence of Sec. 6.1 Eq. 9
# ----------------------------------------------------------------------------
def histogram(x, lo, hi, nbins: int) -> np.ndarray:
    """Counts of x over nbins equal bins of [lo, hi] (uint64); out-of-range values go to the edge bins."""
    a = _f32(x)
    h = np.zeros(nbins, dtype=np.uint64)
    lib().orc_histogram(_fp(a), a.size, ctypes.c_float(float(lo)), ctypes.c_float(float(hi)), int(nbins),
                        h.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
    return h


def kl_divergence(hist_p, hist_q, eps: float = 0.0) -> float:
    """Eq. 9: sum_x P(x) log(P(x) / Q(x)) (natural log) between two histograms over the same bins,
    P the original layer output, Q the quantized one.  Probabilities are (count + eps) /
    (total + eps * nbins); eps = 0 is the plain definition (terms with P = 0 contribute 0, a bin
    with P > 0 and Q = 0 makes the divergence +inf).  The paper gives no smoothing constant."""
    cp = [float(c) for c in hist_p]
    cq = [float(c) for c in hist_q]
    if len(cp) != len(cq) or not cp:
        raise ValueError("histograms must have the same, non-zero number of bins")
    if eps < 0 or math.isnan(eps):
        raise ValueError("eps must be >= 0")
    nb = len(cp)
    tp = sum(cp) + eps * nb
    tq = sum(cq) + eps * nb
    if tp <= 0 or tq <= 0:
        raise ValueError("empty histogram")
    kl = 0.0
    for a, b in zip(cp, cq):
        pa = (a + eps) / tp
        qb_ = (b + eps) / tq
        if pa == 0.0:
            continue
        if qb_ == 0.0:
            return math.inf
        kl += pa * math.log(pa / qb_)
    return kl


# ----------------------------------------------------------------------------
# Sec. 6.3 Eq. 12 (conv + BN folding) and the fusion-aware regrouping of Sec. 6.5
# ----------------------------------------------------------------------------
def bn_fold(w, gamma, var, mean, beta, bias=None):
    """Folded weights A and bias C of Eq. 12 for a weight of shape [channels, ...]."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    ch = w.shape[0]
    inner = w.size // ch
    g, v, m, b = (np.ascontiguousarray(a, dtype=np.float32) for a in (gamma, var, mean, beta))
    bi = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    w_out = np.empty_like(w)
    b_out = np.empty(ch, np.float32)
    lib().orc_bn_fold(_fp(w.reshape(-1)), ch, inner, _fp(g), _fp(v), None if bi is None else _fp(bi),
                      _fp(m), _fp(b), _fp(w_out.reshape(-1)), _fp(b_out))
    return w_out, b_out


def regroup_for_fusion(order, group_id):
    """Sec. 6.5 only allows the list positions of fusion-capable operators to change and gives no
    rule.  Reading taken: layers with the same group id (a conv and the BN / Add / ReLU neighbours it
    fuses with) keep one precision, so a group moves as a block to the position of its most
    sensitive member; inside the block and between blocks the list order is kept."""
    n = len(order)
    if sorted(order) != list(range(n)) or len(group_id) != n:
        raise ValueError("order must be a permutation and group_id one id per layer")
    out, done = [], set()
    for l in order:
        g = group_id[l]
        if g in done:
            continue
        done.add(g)
        out.extend(m for m in order if group_id[m] == g)
    return out
