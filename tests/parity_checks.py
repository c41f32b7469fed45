"""Tensor-by-tensor and element-by-element comparison of a population (the HIP library, or anything with the
same get_params) against the CPU oracle.

Why not one norm per network: a critic is 72 k floats with an L2 norm of about 16, so a head bias (one scalar)
or a whole hidden bias vector that is never updated moves the network's relative L2 error by ~2e-5 and hides
under a 1e-4 bound.  Every comparison here is therefore made per tensor (W1, b1, W2, b2, W3, b3 in the canonical
flat order of a network) and, for single steps from a common state, per element.

Element-wise tolerance of one Adam step (derivation).  Both sides start the step from the same state (initial
state, or the oracle's state rounded to fp32 and written to the device).  The fp32 path's gradient differs from
the fp64 one by rounding: |g_gpu - g_ref| <= E = ETA * (S + FLOOR * largest gradient entry of the layer), S = the
sum over the batch of the absolute values of the terms the entry is a sum of (relu_ties.abs_sums; a head bias is ONE such sum and may cancel to nothing, so its own
size is no scale; asserted when the gradients are exported).  Adam turns that into a parameter difference through
    d(theta)/dg = lr / s * [ (1-b1)/c1 - (m^/s) (g/sqrt(v^)) (1-b2)/c2 ],   s = sqrt(v^) + eps,
whose bracket is bounded by k1 = (1-b1)/c1 + sqrt((1-b2)/c2) (|m^/s| <~ 1, |g|/sqrt(v^) <= sqrt(c2/(1-b2))).  So
    |theta_gpu - theta_ref| <= TOL * max(|theta_ref|, lr) + min(lr * k1 * E / s, 2 lr)
for entries with a history (m or v non-zero before the step).  For fresh entries (m = v = 0 before: the first
step) the update is -lr g / (|g| + eps): it depends on g only through its sign once |g| >> eps (its derivative
eps / (|g| + eps)^2 takes the place of k1 / s above), so an entry is either well determined (|g_ref| >= 2 E:
the sign is safe) or not (masked: only |difference| <= 2 lr is required).  Entries whose sensitivity term exceeds lr / 10 count as masked
as well; the number of masked entries is returned and printed.  Where the oracle's gradient is exactly zero
(units dead on the whole batch) and the entry is fresh, parameter and moments must not change at all.
Targets: t = (1 - tau) t_before + tau theta, so |t_gpu - t_ref| <= 1e-6 |t_ref| + tau * (the bound above).
"""
import numpy as np

TENSORS = ("W1", "b1", "W2", "b2", "W3", "b3")
ETA = 8e-6          # element-wise bound on the gradient's rounding error, relative to the sum of its absolute terms.  The
                    # rigorous bound for the 256- to 448-term fp32 dot products of this path is n 2^-24 = 1.5e-5 .. 2.7e-5
                    # per product (and a gradient entry is several products deep); measured worst on the device: 7.4e-7 at
                    # fan-ins up to 256, 2.8e-6 at 393, 4.4e-6 at 448
FLOOR = 0.05        # ... plus this fraction of ETA times the layer's largest gradient entry: a term whose activation is
                    # nearly zero carries that activation's absolute error, not a relative one (measured on the device:
                    # up to 1.2e-8 of the layer's largest entry beyond 1e-6 * S)
TOL = 1e-4          # one-step parameter tolerance (relative; lr is the floor of the scale)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def tensor_slices(fan_in, fan_out, hidden=(256, 256)):
    """[(name, slice)] of a network's tensors in the canonical flat order (W[in, out] row-major, then b)."""
    sizes = [fan_in] + list(hidden) + [fan_out]
    out, o = [], 0
    for l, (fi, fo) in enumerate(zip(sizes[:-1], sizes[1:])):
        out.append(("W%d" % (l + 1), slice(o, o + fi * fo))); o += fi * fo
        out.append(("b%d" % (l + 1), slice(o, o + fo))); o += fo
    return out, o


def net_shape(net, obs_dim, act_dim, sac=False):
    """(fan_in, fan_out) of 'actor', 'critic1', 'critic2' (also with a t_/m_/v_/g_ prefix)."""
    base = net.split("_")[-1]
    if base == "actor":
        return obs_dim, (2 * act_dim if sac else act_dim)
    return obs_dim + act_dim, 1


def check_tensors(got, ref, net, obs_dim, act_dim, tol, label, sac=False, scale_floor=None, outliers=0, outlier_bound=0.0):
    """Per-tensor relative L2 of one flat network.  The error of tensor T is measured against
    max(||ref_T||, scale_floor * sqrt(n_T)): biases start at zero and stay small, so their own norm is not a
    scale; scale_floor defaults to the network's rms parameter.

    outliers: after free-running steps, up to this many entries per tensor are left out of the norm, each bounded
    by outlier_bound instead.  Adam's first update is -lr sign(g): an entry whose gradient is below the rounding
    error of the fp32 path may start with the other sign and then stays 2 lr away (check_adam_step masks the same
    entries in single steps, where they can be identified).  Returns (worst error / tolerance, entries left out)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    sl, n = tensor_slices(*net_shape(net, obs_dim, act_dim, sac))
    assert got.size == ref.size == n, (label, net, got.size, ref.size, n)
    floor = float(np.sqrt(np.mean(ref * ref))) if scale_floor is None else scale_floor
    worst, left_out = 0.0, 0
    for name, s in sl:
        d = np.abs(got[s] - ref[s])
        scale = max(float(np.linalg.norm(ref[s])), floor * np.sqrt(s.stop - s.start))
        err = float(np.linalg.norm(d))
        if err > tol * scale and outliers:
            order = np.argsort(d)[::-1][:outliers]
            for k in range(1, len(order) + 1):             # leave out as few as needed
                rest = d.copy(); rest[order[:k]] = 0.0
                if float(np.linalg.norm(rest)) <= tol * scale:
                    assert d[order[:k]].max() <= outlier_bound, "%s: %s.%s entry off by %.3e > %.3e" % (
                        label, net, name, d[order[:k]].max(), outlier_bound)
                    err, left_out = float(np.linalg.norm(rest)), left_out + k
                    break
        assert err <= tol * scale, "%s: %s.%s error %.3e > %.1e * %.3e" % (label, net, name, err, tol, scale)
        worst = max(worst, err / (tol * scale) if scale > 0 else 0.0)
    return worst, left_out


class StepReport:
    def __init__(self):
        self.entries = self.masked = self.zero = self.one_sided_zero = 0
        self.tie_units = 0           # hidden units on their kink whose possible flip was allowed for (see tie_envelope)
        self.worst_ratio = 0.0       # worst |difference| / tolerance over unmasked parameter entries
        self.worst_tensor = 0.0      # worst per-tensor relative L2 of parameters (unmasked entries)
        self.worst_grad = 0.0        # worst |g_gpu - g_ref| / (sum of the absolute terms of that entry)
        self.worst_grad_l2 = 0.0

    def __str__(self):
        return ("%d parameter entries compared element by element, %d masked (ill-conditioned Adam update), %d with an "
                "exactly zero gradient unchanged (%d zero on one side only); worst difference / tolerance %.3f, worst per-tensor rel-L2 %.2e; "
                "gradients: worst element error %.2e of the sum of its absolute terms, worst per-tensor rel-L2 %.2e; %d hidden units on their kink allowed for"
                % (self.entries, self.masked, self.zero, self.one_sided_zero, self.worst_ratio, self.worst_tensor, self.worst_grad,
                   self.worst_grad_l2, self.tie_units))


def check_adam_step(rep, label, net, shape, got, ref, before, lr, b1, b2, eps, count, tau=None, tol=TOL, eta=ETA,
                    grad_l2_tol=2e-5, g_scale=None, g_extra=None):
    """One network after one Adam step from a common state.

    got / ref: dicts with flat arrays 'theta', 'm', 'v' (and 'target' when the targets moved, 'g' when exported /
    always for ref); before: dict with the common state 'theta', 'm', 'v' (and 'target').  count: Adam's step
    count of this update.  g_scale: per gradient entry, the sum of the absolute values of its terms (the scale of
    its rounding error); without it the layer's largest gradient entry stands in.  g_extra: per gradient entry, an
    amount added to that error bound (relu_ties.tie_envelope).  Raises AssertionError naming
    the tensor and element; accumulates into rep."""
    sl, n = tensor_slices(*shape)
    f64 = lambda x: np.asarray(x, dtype=np.float64)
    th_g, th_r, th_b = f64(got["theta"]), f64(ref["theta"]), f64(before["theta"])
    m_g, m_r, m_b = f64(got["m"]), f64(ref["m"]), f64(before["m"])
    v_g, v_r, v_b = f64(got["v"]), f64(ref["v"]), f64(before["v"])
    g_r = f64(ref["g"])
    g_g = f64(got["g"]) if got.get("g") is not None else None
    assert th_g.size == th_r.size == g_r.size == n, (label, net, th_g.size, th_r.size, g_r.size, n)
    c1, c2 = 1.0 - b1 ** count, 1.0 - b2 ** count
    k1 = (1.0 - b1) / c1 + np.sqrt((1.0 - b2) / c2)
    layer_max = {}                                         # a bias gradient is a sum of the same dz terms as its layer's
    for name, s in sl:                                     # weight gradient and may cancel to nothing (a head bias is
        layer_max[name[1]] = max(layer_max.get(name[1], 0.0), float(np.abs(g_r[s]).max()))   # ONE such sum): scale per layer
    for name, s in sl:
        tag = "%s: %s.%s" % (label, net, name)
        g = g_r[s]; gmax = layer_max[name[1]]
        e_g = eta * gmax if g_scale is None else eta * np.asarray(g_scale, dtype=np.float64)[s] + FLOOR * eta * gmax
        if g_extra is not None:
            e_g = e_g + np.asarray(g_extra, dtype=np.float64)[s]
        if g_g is not None:
            dg = np.abs(g_g[s] - g)
            worst = int((dg - e_g).argmax())
            assert np.all(dg <= e_g), "%s gradient element %d: %.6e vs %.6e (largest of the layer %.3e, allowed difference %.3e)" % (
                tag, worst, g_g[s][worst], g[worst], gmax, np.broadcast_to(e_g, dg.shape)[worst])
            if gmax > 0.0:
                rep.worst_grad = max(rep.worst_grad, float((dg / np.maximum(e_g, 1e-300)).max()) * eta)
                # per-tensor norm; a tensor whose entries cancel to under 10 % of their terms (a head bias can) is
                # measured against those terms
                scale = float(np.linalg.norm(g))
                if g_scale is not None:
                    scale = max(scale, 0.1 * float(np.linalg.norm(np.asarray(g_scale, dtype=np.float64)[s])))
                extra = float(np.linalg.norm(np.asarray(g_extra, dtype=np.float64)[s])) if g_extra is not None else 0.0
                e = max(float(np.linalg.norm(g_g[s] - g)) - extra, 0.0) / scale
                if g.size >= 8:                              # (a one-entry tensor has had its whole test element-wise)
                    rep.worst_grad_l2 = max(rep.worst_grad_l2, e)
                    assert e <= grad_l2_tol, "%s gradient rel-L2 %.3e" % (tag, e)
            # exactly zero on one side only: a unit dead on the whole batch for one side and, through a pre-activation
            # within rounding of zero, alive with a negligible value for the other (the difference is inside e_g,
            # checked above); such entries are rare and are treated as undetermined below
            one_sided = (g == 0.0) != (g_g[s] == 0.0)
            assert int(one_sided.sum()) <= 8, "%s: %d entries are exactly zero on one side only" % (tag, int(one_sided.sum()))
            rep.one_sided_zero += int(one_sided.sum())
        fresh = (m_b[s] == 0.0) & (v_b[s] == 0.0)
        sdev = np.sqrt(v_r[s] / c2) + eps
        sens = lr * k1 * e_g / sdev
        # fresh entries: d/dg [g / (|g| + eps)] = eps / (|g| + eps)^2, which matters only where |g| is of the order of eps
        sens_fresh = lr * eps * e_g / (np.maximum(np.abs(g) - e_g, 0.0) + eps) ** 2
        sens = np.where(fresh, sens_fresh, sens)
        base = tol * np.maximum(np.abs(th_r[s]), lr)
        determined = np.where(fresh, np.abs(g) >= 2.0 * e_g, True) & (sens <= 0.1 * lr)
        zero = fresh & (g == 0.0)
        if g_g is not None:
            zero = zero & (g_g[s] == 0.0)
            determined = determined & ~one_sided
        determined = determined | zero
        tol_el = base + np.minimum(sens, 2.0 * lr)
        tol_el = np.where(determined, tol_el, 2.0 * lr * (1.0 + 1e-3) + 1e-6 * np.abs(th_r[s]))
        d = np.abs(th_g[s] - th_r[s])
        bad = d > tol_el
        assert not bad.any(), "%s element %d: %.8e vs %.8e, difference %.3e > %.3e (g_ref %.3e of max %.3e, lr %.3e, %s)" % (
            tag, int(bad.argmax()), th_g[s][bad.argmax()], th_r[s][bad.argmax()], d[bad.argmax()], tol_el[bad.argmax()],
            g[bad.argmax()], gmax, lr, "fresh" if fresh[bad.argmax()] else "with history")
        # exactly zero gradient on a fresh entry: nothing may change
        if zero.any():
            b32 = th_b[s].astype(np.float32).astype(np.float64)
            assert np.array_equal(th_g[s][zero], b32[zero]), "%s: parameter moved under an exactly zero gradient" % tag
            assert not m_g[s][zero].any() and not v_g[s][zero].any(), "%s: moments moved under a zero gradient" % tag
        keep = determined & ~zero
        rep.entries += int(keep.sum()); rep.masked += int((~determined).sum()); rep.zero += int(zero.sum())
        if keep.any():
            rep.worst_ratio = max(rep.worst_ratio, float((d[keep] / tol_el[keep]).max()))
            err = float(np.linalg.norm(d[keep]))
            scale = max(float(np.linalg.norm(th_r[s][keep])), lr * np.sqrt(keep.sum()))
            rep.worst_tensor = max(rep.worst_tensor, err / scale)
            assert err <= tol * scale + float(np.linalg.norm(np.minimum(sens, 2.0 * lr)[keep & ~fresh])), \
                "%s per-tensor error %.3e (scale %.3e)" % (tag, err, scale)
        # moments, all entries: m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2
        dm = np.abs(m_g[s] - m_r[s])
        tm = 2e-5 * np.abs(m_r[s]) + (1.0 - b1) * e_g
        assert np.all(dm <= tm), "%s first moment element %d: %.6e vs %.6e" % (tag, int((dm - tm).argmax()),
                                                                           m_g[s][(dm - tm).argmax()], m_r[s][(dm - tm).argmax()])
        dv = np.abs(v_g[s] - v_r[s])
        tv = 4e-5 * np.abs(v_r[s]) + (1.0 - b2) * (2.0 * np.abs(g) * e_g + e_g ** 2)
        assert np.all(dv <= tv), "%s second moment element %d: %.6e vs %.6e" % (tag, int((dv - tv).argmax()),
                                                                            v_g[s][(dv - tv).argmax()], v_r[s][(dv - tv).argmax()])
        if tau is not None:
            t_g, t_r = f64(got["target"])[s], f64(ref["target"])[s]
            dt = np.abs(t_g - t_r)
            tt = 1e-6 * np.abs(t_r) + tau * tol_el + 1e-12
            assert np.all(dt <= tt), "%s target element %d: %.8e vs %.8e (tolerance %.3e)" % (
                tag, int((dt - tt).argmax()), t_g[(dt - tt).argmax()], t_r[(dt - tt).argmax()], tt[(dt - tt).argmax()])


def check_unchanged(label, net, got, before):
    """A network that takes no update in this step (delayed actor, targets between delayed steps): bit-unchanged."""
    for k, arr in got.items():
        if arr is None or k == "g":
            continue
        b32 = np.asarray(before[k], dtype=np.float64).astype(np.float32)
        assert np.array_equal(np.asarray(arr, dtype=np.float32), b32), "%s: %s %s changed in a step without its update" % (label, net, k)
