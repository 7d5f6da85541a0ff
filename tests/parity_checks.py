"""Comparison of a flat parameter / gradient vector from the HIP path with the oracle's, tensor by
tensor (test helper: no arithmetic of the method).

Three bounds per tensor, all of which must hold:
  L2           |got - ref|_2 <= tol * |ref|_2                      (the contract's relative error)
  element-wise |got - ref| <= tol * C_RMS * max(rms(ref), |ref|)   (every entry: a relative bound for
                                                                    the large entries of a heavy-tailed
                                                                    tensor, an absolute one -- a small
                                                                    fraction of the tensor's typical
                                                                    entry -- for the others)
  conditioned  when `scale` is given (for every entry the sum of the absolute values of the terms
               the chain rule adds up for it, from oracle.matrix_form.grad_error_scale): a tensor
               whose entries are sums that cancel -- a bias gradient over two classes and two rows --
               has no meaningful relative error, so both bounds above are taken against
               max(|ref|_2, rho * |scale|_2) and max(rms(ref), rho * rms(scale)), and in addition
               every entry obeys |got - ref| <= tol_scale * scale, the textbook forward error bound
               of a sum evaluated in floating point.
"""
import numpy as np

import hb_inputs as hi

C_RMS = 8.0     # element-wise bound, in units of tol * rms(ref)
RHO = 1e-2      # a tensor counts as cancelled when |ref| < RHO * |scale| (fp32: tol * RHO = 1e-6, 16 roundings)
RHO_BF16 = 0.1  # bf16 storage: tol * RHO = 2e-3 = 2^-9, one bf16 rounding of every term


def tensors(dims):
    """[(name, slice)] per parameter tensor of the flat layout."""
    out = []
    for l, (wo, bo) in enumerate(hi.param_offsets(dims), start=1):
        out.append((f"W{l}", slice(wo, wo + dims[l] * dims[l - 1])))
        out.append((f"b{l}", slice(bo, bo + dims[l])))
    return out


def tensor_errors(dims, got, ref, scale=None):
    """Per tensor: dict(l2, l2_ref, rms_ref, max_abs, arg, l2_scale, rms_scale, max_over_scale)."""
    rep = {}
    for name, sl in tensors(dims):
        r = np.asarray(ref[sl], dtype=np.float64)
        g = np.asarray(got[sl], dtype=np.float64)
        e = np.abs(g - r)
        d = dict(l2=float(np.linalg.norm(e)), l2_ref=float(np.linalg.norm(r)),
                 rms_ref=float(np.sqrt(np.mean(r * r))), max_abs=float(e.max()), arg=int(e.argmax()),
                 finite=bool(np.isfinite(g).all()), err=e, absref=np.abs(r))
        if scale is not None:
            s = np.asarray(scale[sl], dtype=np.float64)
            d.update(l2_scale=float(np.linalg.norm(s)), rms_scale=float(np.sqrt(np.mean(s * s))),
                     max_over_scale=float(np.max(e / np.maximum(s, 1e-300))))
        rep[name] = d
    return rep


def assert_close(dims, got, ref, tol, what, scale=None, tol_scale=None, scale_factor=1.0, abs_floor=0.0,
                 ref_rounding=0.0, rho=RHO):
    """scale_factor multiplies `scale` and ref_rounding * |ref| is added to the per-entry bound:
    when parameters after a step are compared, their error is lr times the gradient's plus one
    rounding of the parameter itself (scale_factor = lr, ref_rounding = one unit in the last place
    of the storage type)."""
    rep = tensor_errors(dims, got, ref, scale)
    bad = []
    for name, d in rep.items():
        if not d["finite"]:
            bad.append(f"{name}: non-finite values")
            continue
        l2_den, rms_den = max(d["l2_ref"], abs_floor), max(d["rms_ref"], abs_floor)
        if scale is not None:
            l2_den = max(l2_den, rho * scale_factor * d["l2_scale"])
            rms_den = max(rms_den, rho * scale_factor * d["rms_scale"])
        if l2_den == 0.0:
            if d["l2"] != 0.0:
                bad.append(f"{name}: reference is zero, got |.|_2 = {d['l2']:.3e}")
            continue
        if not d["l2"] <= tol * l2_den:
            bad.append(f"{name}: L2 error {d['l2'] / l2_den:.3e} of the reference (> {tol:g})")
        over = d["err"] > tol * C_RMS * np.maximum(rms_den, d["absref"])
        if over.any():
            i = int(np.argmax(np.where(over, d["err"], 0.0)))
            bad.append(f"{name}: {int(over.sum())} entries off by more than {tol * C_RMS:g} x max(rms, |entry|); "
                       f"worst entry {i}: {d['err'][i] / rms_den:.3e} rms, reference {d['absref'][i] / rms_den:.3e} rms")
    if scale is not None and tol_scale is not None:
        for name, sl in tensors(dims):
            r = np.asarray(ref[sl], dtype=np.float64)
            e = np.abs(np.asarray(got[sl], dtype=np.float64) - r)
            lim = tol_scale * scale_factor * np.asarray(scale[sl], dtype=np.float64) + ref_rounding * np.abs(r)
            over = np.nonzero(e > lim)[0]
            if over.size:
                i = over[np.argmax((e / np.maximum(lim, 1e-300))[over])]
                bad.append(f"{name}: {over.size} entries beyond {tol_scale:g} x the sum of their absolute terms, "
                           f"worst entry {i}: error {e[i]:.3e}, bound {lim[i]:.3e}")
    assert not bad, f"{what}: " + "; ".join(bad) + " | all: " + ", ".join(
        f"{k} L2 {v['l2'] / max(v['l2_ref'], 1e-300):.1e} max/rms {v['max_abs'] / max(v['rms_ref'], 1e-300):.1e}"
        for k, v in rep.items())
