"""Helpers shared by the GPU parity tests: build a device stage (through the C ABI binding) and
the CPU oracle from the same seeded inputs, and compare them tensor by tensor."""
import numpy as np

import zb_inputs
from oracle import optimizer as O
from oracle.stage import StageOracle, PARAM_ORDER

TOL = {"fp32": 1e-4, "bf16": 2e-2}   # max relative Frobenius error per tensor: fp32 arithmetic, bf16 storage with fp32 accumulation


def rel_fro(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


# Element-wise bound beside the Frobenius one.  The error of a device tensor against the fp64 oracle is the sum
# of many independent roundings (bf16 storage of every intermediate, fp32 accumulation), so its entries scatter
# around zero with a standard deviation of about (relative Frobenius error) x rms(reference).  They are not
# identically distributed - a token's row carries the factor 1/sigma of its LayerNorm, an input feature's row of
# a weight gradient the magnitude of that feature - so the largest of the up to 1e8 entries of a tensor lies
# further out than the 6 standard deviations of a normal sample: up to 7 were seen at the workloads' shapes, and
# the bound is put at 10.  On top comes the final rounding of the entry itself to the storage type, half an ulp
# of ITS OWN magnitude (2^-9 relative for bf16; large entries of a tensor are several times its rms).  Hence
#     |a - b| <= ELEM_K * tol * rms(b) + ULP[dtype] * |b|     for every entry
# (0.2 rms(b) for bf16).  A wrong column, a dropped bias or a single wrong gradient entry is off by about
# rms(b) or more, five times the bound, while the Frobenius norm alone would let it pass.
ELEM_K = 10.0
ULP = {"fp32": 2.0 ** -22, "bf16": 2.0 ** -8}


def elem_excess(a, b, tol, dtype, by_row=False):
    """Largest |a - b| / (ELEM_K * tol * rms(b) + ULP * |b|) over the entries (<= 1 passes).  rms is taken over
    the entries of b that hold something; with by_row, row by row of a matrix whose rows are sums of different
    numbers of terms (a token table's gradient: a frequent id's row adds a hundred rows, a rare one's a single
    one, most none - those must be exactly zero)."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    if not b.size:
        return 0.0
    if by_row and b.ndim == 2:
        live = b != 0
        n = np.maximum(live.sum(axis=1), 1)
        rms = np.sqrt((b * b).sum(axis=1) / n)[:, None]
    else:
        live = b[b != 0]
        rms = float(np.sqrt(np.mean(live * live))) if live.size else 0.0
    bound = np.maximum(ELEM_K * tol * rms + ULP[dtype] * np.abs(b), 1e-300)
    return float(np.max(np.abs(a - b) / bound))


def check_tensor(label, a, b, tol, dtype, by_row=False):
    """Both bounds; returns (relative Frobenius error, element-wise excess)."""
    e = rel_fro(a, b)
    assert e <= tol, f"{label}: rel fro {e:.3e} > {tol}"
    x = elem_excess(a, b, tol, dtype, by_row)
    assert x <= 1.0, f"{label}: an entry is off by {x:.2f} x the element-wise bound"
    return e, x


def check_second_moment(label, v_dev, v_ref, tol):
    """Adam's v is quadratic in the gradients: twice their relative error in the Frobenius norm; entry by
    entry its error grows with the entry itself (dv = 2 g dg), so the element-wise bound is applied to
    sqrt(v), which is linear in the gradients."""
    v_dev = np.asarray(v_dev, np.float64)
    v_ref = np.asarray(v_ref, np.float64)
    e = rel_fro(v_dev, v_ref)
    assert e <= 2 * tol, f"{label}: rel fro {e:.3e} > {2 * tol}"
    assert (v_dev >= 0).all(), f"{label}: negative second moment"
    x = elem_excess(np.sqrt(v_dev), np.sqrt(v_ref), tol, "fp32")
    assert x <= 1.0, f"{label}: sqrt(v) of an entry is off by {x:.2f} x the element-wise bound"
    return e, x


def check_delta_theta(label, before, after, ref_before, ref_after, ref_v, tol):
    """The parameter UPDATE of one optimizer step against the oracle's update.  At the workloads' learning
    rate a step moves a parameter by far less than the tolerance on the parameter itself, so comparing theta
    alone cannot tell a step from no step.  Adam's update of an entry is lr * m / sqrt(v): where the entry's
    gradients have all been small against the rounding noise of their tensors (relative to the tensor's rms,
    not to the entry), m and sqrt(v) are both noise and the update flips sign whatever the kernel does (the
    first step is exactly lr * sign(g)).  Such entries are left out: kept are those whose second moment v
    (the oracle's, after the step) is at least 1/16 of the tensor's mean v, i.e. whose gradients were at
    least a quarter of the rms - about four fifths of a tensor with normal entries (at least the larger half,
    whatever the distribution).  Mean and median are taken over the entries that received a gradient at all
    (most rows of an embedding table do not, in one iteration)."""
    v = np.asarray(ref_v, np.float64).reshape(-1)
    seen = v[v > 0]
    assert seen.size > 0, f"{label}: no entry received a gradient"
    keep = v >= min(np.mean(seen) / 16.0, np.median(seen))
    d_dev = (np.asarray(after, np.float64).reshape(-1) - np.asarray(before, np.float64).reshape(-1))[keep]
    d_ref = (np.asarray(ref_after, np.float64).reshape(-1) - np.asarray(ref_before, np.float64).reshape(-1))[keep]
    assert np.linalg.norm(d_ref) > 0, f"{label}: the oracle did not move"
    e = rel_fro(d_dev, d_ref)
    assert e <= tol, f"{label}: update rel fro {e:.3e} > {tol}"
    return e


def hyper(w):
    return O.Hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.adam_eps, weight_decay=w.weight_decay, clip=w.clip)


def make_device_stage(w, m=None, pools=None, journal=True, group_w=True, fuse_bw=False):
    import paper_2401_10241_amd as zb
    m = m or w.m
    pb, pw, fl = pools or zb.schedule_stash_need(w.p, w.stage, m, w.kind)
    return zb.Stage(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, mb_size=w.mb_size,
                    dtype=w.dtype, max_microbatches=m, max_pending_b=pb, max_pending_w=pw, max_inflight=fl,
                    journal=journal, group_w=group_w, fuse_bw=fuse_bw, ln_eps=w.ln_eps, lr=w.lr, beta1=w.beta1, beta2=w.beta2,
                    adam_eps=w.adam_eps, weight_decay=w.weight_decay, clip=w.clip)


def make_oracle(w, params):
    return StageOracle(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, mb_size=w.mb_size,
                       dtype=w.dtype, ln_eps=w.ln_eps, hyper=hyper(w), params=params)


def load_iteration(w, it, m, dev=None, orc=None, mbs=None):
    """Feeds the same seeded X_k, dY_k to the device stage and/or the oracle."""
    import paper_2401_10241_amd as zb
    for k in (range(m) if mbs is None else mbs):
        X = zb_inputs.stage_input(w, it, k)
        dY = zb_inputs.upstream_grad(w, it, k)
        if dev is not None:
            dev.set_tensor(zb.T_INPUT_X, 0, k, X)
            dev.set_tensor(zb.T_INPUT_DY, 0, k, dY)
        if orc is not None:
            orc.set_input(k, X)
            orc.set_upstream_grad(k, dY)


def _dtype_of(dev):
    return "bf16" if dev.cfg.dtype == 1 else "fp32"


WORST_ELEM = [0.0]   # largest element-wise excess seen in this process (printed by the tests)


def compare_grads(dev, orc, tol, what=None):
    """Accumulated gradients of all 12 tensors of every layer: Frobenius and element-wise bounds (gradients are
    stored in fp32 for both data types, so the last-rounding term is fp32's)."""
    import paper_2401_10241_amd as zb
    worst = 0.0
    got = dev.get_group(zb.T_GRAD if what is None else what)
    for l in range(len(got)):
        for name in PARAM_ORDER:
            e, x = check_tensor(f"grad layer {l} {name}", got[l][name], orc.grads[l][name], tol, "fp32")
            worst = max(worst, e)
            WORST_ELEM[0] = max(WORST_ELEM[0], x)
    return worst


def compare_outputs(dev, orc, m, tol, mbs=None):
    import paper_2401_10241_amd as zb
    worst = 0.0
    dt = _dtype_of(dev)
    for k in (range(m) if mbs is None else mbs):
        e, x = check_tensor(f"Y[{k}]", dev.get_tensor(zb.T_OUTPUT_Y, 0, k), orc.Y[k], tol, dt)
        e2, x2 = check_tensor(f"dX[{k}]", dev.get_tensor(zb.T_OUTPUT_DX, 0, k), orc.dX[k], tol, dt)
        worst = max(worst, e, e2)
        WORST_ELEM[0] = max(WORST_ELEM[0], x, x2)
    return worst
