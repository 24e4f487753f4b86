"""Runs the HIP library through its C ABI (via the ctypes binding) on workloads
given as numpy arrays, and returns numpy arrays.  Used by the `gpu` tests only."""
import os

import numpy as np
import torch

import paper_2110_09524_amd as pk

RTOL = 1e-4   # the stated fp32 tolerance: |gpu - oracle| <= ATOL + RTOL * |oracle|
ATOL = 1e-5


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def empty(shape, dtype=torch.float32):
    # poison outputs so an element the kernel never writes cannot pass by luck
    t = torch.empty(shape, dtype=dtype, device="cuda")
    if dtype == torch.float32:
        t.fill_(float("nan"))
    else:
        t.fill_(-12345)
    return t


def workspace(nbytes):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")


# Every comparison leaves one record here: how many entries miss the literal bound
# ATOL + RTOL * |oracle| (no scaling of the absolute term) and by what factor at worst.
# tests/conftest.py writes the records to tolerance_report.jsonl at the end of a run.
LITERAL_LOG = []


def _log_literal(name, err, ref, scaled, rtol, atol):
    lit = ATOL + RTOL * np.abs(ref)
    ratio = err / lit
    miss = ratio > 1.0
    LITERAL_LOG.append(dict(
        test=os.environ.get("PYTEST_CURRENT_TEST", "").split(" ")[0], tensor=name, entries=int(err.size),
        scaled_bound=bool(scaled), widened=bool(rtol != RTOL or atol != ATOL),
        literal_misses=int(miss.sum()), worst_ratio=float(ratio.max()) if err.size else 0.0,
        rms_ref=float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0))


# Filled by the randomised sweep only, with tensor names that take the row-scaled absolute term
# there.  Its layers are up to 1024 columns wide with operands of order 1 and rows that hear from
# most of the graph, so an entry of gx = dz w^T is a dot product of up to 1024 terms of both signs
# (same class as the product gradients), and the unnormalised GMM sum of a hub row is the hub-row
# class; under the literal bound 62 of 2949 such random cases miss it, by 3.7x at worst, in exactly
# these tensors.  The workload tests keep gx literal.
ROW_SCALED_IN_SWEEP = set()


def assert_close(name, got, ref, rtol=RTOL, atol=ATOL, reduce_scale=False, row_scale=False):
    """Element-wise |got - ref| <= atol_eff + rtol |ref|; atol_eff = atol (the literal bound) unless:

    reduce_scale=True, for the gradients that are matrix products or sums over ALL vertices or
    edges with terms of both signs (gw, gw_fc, gtheta, gphi, ga_l, ga_r): fp32 rounding there is
    proportional to the partial sums, not to the (possibly cancelled) entry, so the absolute term
    scales with the tensor's rms value: atol_eff = atol * max(1, rms(ref)).

    row_scale=True, for unnormalised sums over the ~10^4 in-edges of a hub row, and for the
    gradients of the deliberately ill-conditioned large-score case: atol_eff[u] = atol *
    max(1, max_j |ref[u, j]|).

    tests/test_fp32_summation_bounds.py shows on the CPU that a plain fp32 evaluation in the
    oracle's own order misses the literal bound in exactly these cases, by the same factors.
    Every comparison is also logged against the literal bound (LITERAL_LOG).
    """
    if name in ROW_SCALED_IN_SWEEP:
        row_scale = True
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values in the GPU result"
    a = atol
    if reduce_scale and ref.size:
        a = atol * max(1.0, float(np.sqrt(np.mean(ref * ref))))
    if row_scale and ref.ndim == 2 and ref.size:
        a = atol * np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True))
    err = np.abs(got - ref)
    tol = a + rtol * np.abs(ref)
    _log_literal(name, err, ref, reduce_scale or row_scale, rtol, atol)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(
            f"{name}: {int(bad.sum())}/{bad.size} entries out of tolerance; worst at {i}: "
            f"gpu={got[i]:.9g} oracle={ref[i]:.9g} err={err[i]:.3g} tol={tol[i]:.3g}")


def gat_kink_masks(indptr, fwd, tol=1e-5):
    """LeakyReLU' jumps at a raw score of exactly 0, and the fp32 path decides the sign
    from scores that carry ~1e-6 of rounding.  An edge whose fp64 raw score lies within
    `tol` of 0 may therefore legitimately take either slope; what depends on that choice
    is excluded from the comparison: (vertex, head) entries of the destination-side sums
    of a row holding such an edge, and the input-gradient rows of its two endpoints.
    Returns (amb_vh [n, heads] bool, amb_vertex [n] bool)."""
    amb_e = np.abs(fwd["M0"]) < tol
    n = indptr.shape[0] - 1
    # The exclusion must stay an exception.  Scores of order 1 land within 1e-5 of zero at a rate
    # of about 1e-5, so: at most one score in 10^4, and at most 1 % of the vertices masked; on
    # small dense test graphs (a few hundred vertices, 10^5 .. 10^6 scores) up to 10 % of the rows.
    n_amb = int(amb_e.sum())
    assert n_amb <= max(4, amb_e.size // 10_000), f"{n_amb} of {amb_e.size} scores sit on the LeakyReLU kink"
    rows_masked = 2 * int(amb_e.any(axis=1).sum())
    assert rows_masked <= max(4, n // 100 if n >= 5000 else n // 10), \
        f"{rows_masked} of {n} rows would be masked: the mask would hide the test"
    amb_vh = np.zeros((n, amb_e.shape[1]), dtype=bool)
    amb_vertex = np.zeros(n, dtype=bool)
    if amb_e.any():
        e_idx, h_idx = np.nonzero(amb_e)
        amb_vh[fwd["dst"][e_idx], h_idx] = True
        amb_vertex[fwd["dst"][e_idx]] = True
        amb_vertex[fwd["src"][e_idx]] = True
    return amb_vh, amb_vertex


def run_gat(c, backward=True, want_gx=True, graph=None, stash=True, alpha_stash=False):
    """stash=True: the forward call writes t and sg and the backward call uses them;
    stash=False: the backward call recomputes them over the in-edges.
    alpha_stash=True: the per-edge softmax values are stored after the forward call and the
    backward call reads them back (gnn_gat_stash_alpha + gnn_gat_bwd_stashed)."""
    n, fin, H, F = c["n"], c["fin"], c["heads"], c["f"]
    HF = H * F
    indptr, indices = dev(c["indptr"]), dev(c["indices"])
    g = graph or pk.Graph(indptr, indices)
    x, w, a_l, a_r = dev(c["x"]), dev(c["w"]), dev(c["a_l"]), dev(c["a_r"])
    z, out = empty((n, HF)), empty((n, HF))
    el, er, m, d = (empty((n, H)) for _ in range(4))
    ws = workspace(pk.gnn_gat_workspace_bytes(g, fin, H, F))
    t = empty((n, HF)) if stash else None
    sg = empty((n, H)) if stash else None
    pk.gnn_gat_fwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, ws)
    res = dict(z=z, el=el, er=er, m=m, d=d, out=out)
    if stash:
        res.update(t=t, sg=sg)
    alpha_t = None
    if alpha_stash:
        alpha_t = empty((max(len(c["indices"]), 1), H))
        pk.gnn_gat_stash_alpha(g, H, F, c["slope"], el, er, m, d, alpha_t)
        res["alpha_t"] = alpha_t
    if backward:
        gout = dev(c["gout"])
        ws.fill_(0xFF)      # nothing may survive in the workspace between the two calls
        gx = empty((n, fin)) if want_gx else None
        gw, ga_l, ga_r = empty((fin, HF)), empty((H, F)), empty((H, F))
        if alpha_stash:
            pk.gnn_gat_bwd_stashed(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg,
                                   alpha_t, gout, gx, gw, ga_l, ga_r, ws)
        else:
            pk.gnn_gat_bwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, gout,
                           gx, gw, ga_l, ga_r, ws)
        res.update(gw=gw, ga_l=ga_l, ga_r=ga_r)
        if want_gx:
            res["gx"] = gx
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}


def run_edgeconv(c, backward=True, gout=None):
    n, fin, fout = c["n"], c["fin"], c["fout"]
    indptr, indices = dev(c["indptr"]), dev(c["indices"])
    g = pk.Graph(indptr, indices)
    x, theta, phi = dev(c["x"]), dev(c["theta"]), dev(c["phi"])
    ws = workspace(pk.gnn_edgeconv_workspace_bytes(g, fin, fout))
    pq, out = empty((n, 2 * fout)), empty((n, fout))
    argmax = empty((n, fout), torch.int32)
    pk.gnn_edgeconv_fwd(g, fin, fout, x, theta, phi, pq, out, argmax, ws)
    res = dict(pq=pq, out=out, argmax=argmax)
    if backward:
        go = dev(c["gout"] if gout is None else gout, torch.float32)
        gx, gtheta, gphi = empty((n, fin)), empty((fin, fout)), empty((fin, fout))
        pk.gnn_edgeconv_bwd(g, fin, fout, x, theta, phi, argmax, go, gx, gtheta, gphi, ws)
        res.update(gx=gx, gtheta=gtheta, gphi=gphi)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}


def run_gmm(c, backward=True, fwd_workspace=True):
    """fwd_workspace=False: the forward call gets no workspace and projects before it aggregates
    whatever the widths are (with one it aggregates first when the input rows are narrower)."""
    n, fin, fout, K = c["n"], c["fin"], c["fout"], c["k"]
    indptr, indices = dev(c["indptr"]), dev(c["indices"])
    g = pk.Graph(indptr, indices)
    x, w_fc, cc = dev(c["x"]), dev(c["w_fc"]), dev(c["c"])
    mu, inv_sigma = dev(c["mu"]), dev(c["inv_sigma"])
    hk, out = empty((n, K * fout)), empty((n, fout))
    ws = workspace(pk.gnn_gmm_workspace_bytes(g, fin, fout, K))
    pk.gnn_gmm_fwd(g, fin, fout, K, x, w_fc, cc, mu, inv_sigma, hk, out, ws if fwd_workspace else None)
    res = dict(hk=hk, out=out)
    if backward:
        gout = dev(c["gout"])
        ws.fill_(0xFF)      # nothing may survive in the workspace between the two calls
        gx, gw_fc = empty((n, fin)), empty((fin, K * fout))
        gmu, gis = empty((K, 2)), empty((K, 2))
        pk.gnn_gmm_bwd(g, fin, fout, K, x, w_fc, cc, mu, inv_sigma, hk, gout, gx, gw_fc, gmu, gis, ws)
        res.update(gx=gx, gw_fc=gw_fc, gmu=gmu, ginv_sigma=gis)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}


def run_gcn(c, backward=True, want_gx=True, graph=None):
    n, fin, fout = c["n"], c["fin"], c["fout"]
    indptr, indices = dev(c["indptr"]), dev(c["indices"])
    g = graph or pk.Graph(indptr, indices)
    x, w, c_src, c_dst = dev(c["x"]), dev(c["w"]), dev(c["c_src"]), dev(c["c_dst"])
    zs, out = empty((n, fout)), empty((n, fout))
    pk.gnn_gcn_fwd(g, fin, fout, x, w, c_src, c_dst, zs, out)
    res = dict(zs=zs, out=out)
    if backward:
        ws = workspace(pk.gnn_gcn_workspace_bytes(g, fin, fout))
        ws.fill_(0xFF)
        gx = empty((n, fin)) if want_gx else None
        gw = empty((fin, fout))
        pk.gnn_gcn_bwd(g, fin, fout, x, w, c_src, c_dst, dev(c["gout"]), gx, gw, ws)
        res["gw"] = gw
        if want_gx:
            res["gx"] = gx
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}
