"""Shared comparison code of the GPU parity tests: HIP library output vs the float64 oracle.

Bars (from the build's stated tolerances): top-k indices and |V_k| bit-exact; floats within
rel 1e-5 for fp32 logits and rel 1e-3 for bf16 logits, the same figure taken as an absolute
bound for log-domain outputs; masks exact except where the uniform lies within the float
tolerance of the acceptance probability (there either decision is valid and the oracle's batch
stage is re-run with the decision the GPU took).
"""
import numpy as np
import torch

from oracle import obrs_oracle as orc
from paper_2602_06107_amd import obrs
from paper_2602_06107_amd import workloads as wl

TOL = {torch.float32: 1e-5, torch.bfloat16: 1e-3}
MASK_BAND = 1e-5


def run_oracle(w, n_threads=0, rows=None):
    """Oracle over all rows (or the given row indices) of a workload, on exact copies of its bits."""
    sel = slice(None) if rows is None else torch.as_tensor(rows, device=w.actor.device)
    a = wl.logits_to_numpy(w.actor[sel])
    p = wl.logits_to_numpy(w.policy[sel])
    x = w.sampled_ids[sel].cpu().numpy()
    u = w.uniforms[sel].cpu().numpy()
    return orc.rows(a, p, x, u, w.lam, w.k, n_threads=n_threads)


def _close(got, want, rel, what, abs_tol=0.0):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    same = got == want                       # also covers matching infinities
    with np.errstate(invalid="ignore"):
        err = np.where(same, 0.0, np.abs(got - want))
        bound = np.where(same, 0.0, rel * np.abs(want) + abs_tol)
    bad = ~(err <= bound)
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst index "
                           f"{int(np.argmax(err - bound))}: got {got.flat[np.argmax(err - bound)]!r} "
                           f"want {want.flat[np.argmax(err - bound)]!r}")


def host_outputs(buf):
    """Every output tensor of a call copied to the host once (for checks that go through the batch in pieces)."""
    return {n: t.cpu().numpy() for n, t in buf.tensors.items() if n != "stats"}


def check_rows(buf, w, R, rows=None, flags=0, tol=None, stored=False, host=None):
    """Per-row outputs of the HIP path against oracle rows R (for all rows or the sampled ones).
    stored=True: the stored-actor form, where the actor list is an input and is not written.
    host: the outputs as host_outputs(buf) returned them (else they are copied here)."""
    tol = TOL[w.actor.dtype] if tol is None else tol
    idx = np.arange(w.T) if rows is None else np.asarray(rows)
    o = R.out
    valid = o["valid"] == 1
    host = host_outputs(buf) if host is None else host
    g = {n: a[idx] for n, a in host.items()}

    # padding rows: zeros, ids -1
    if (~valid).any():
        for n in ("accept_prob", "logq", "logp", "logratio", "z_approx"):
            assert np.all(g[n][~valid] == 0.0), n
        assert np.all(g["mask"][~valid] == 0)
        assert np.all(g["topk_policy"][~valid] == -1)
        assert stored or np.all(g["topk_actor"][~valid] == -1)

    v = valid
    if not stored:
        np.testing.assert_array_equal(g["topk_actor"][v], R.topk_q[v], err_msg="top-k(q) ids")
    np.testing.assert_array_equal(g["topk_policy"][v], R.topk_p[v], err_msg="top-k(p) ids")
    np.testing.assert_array_equal(g["union_size"][v], o["union_size"][v], err_msg="|V_k|")
    _close(g["logq"][v], o["logq_x"][v], 0.0, "log q(x)", abs_tol=tol)
    _close(g["logp"][v], o["logp_x"][v], 0.0, "log p(x)", abs_tol=tol)
    _close(g["logratio"][v], o["logratio"][v], 0.0, "log ratio", abs_tol=tol)
    _close(g["accept_prob"][v], o["accept"][v], tol, "a(x)")
    _close(g["z_approx"][v], o["z_approx"][v], tol, "Z_approx")
    if flags & obrs.JP_FLAG_EXACT_Z:
        _close(g["z_exact"][v], o["z_exact"][v], tol, "Z_exact")
    if flags & obrs.JP_FLAG_DISTILL_KL:
        _close(g["distill_kl"][v], o["kl_p_q"][v], tol, "KL(p||q)", abs_tol=tol)
    if flags & obrs.JP_FLAG_TOPK_LOGPROBS:
        p64 = wl.logits_to_float64(w.policy[torch.as_tensor(idx, device=w.actor.device)])
        tp = np.where(valid[:, None], R.topk_p, 0).astype(np.int64)
        want_p = np.take_along_axis(p64, tp, 1) - o["lse_p"][:, None]
        _close(g["topk_policy_logp"][v], want_p[v], 0.0, "top-k log p", abs_tol=tol)
        if not stored:
            a64 = wl.logits_to_float64(w.actor[torch.as_tensor(idx, device=w.actor.device)])
            tq = np.where(valid[:, None], R.topk_q, 0).astype(np.int64)
            want_q = np.take_along_axis(a64, tq, 1) - o["lse_q"][:, None]
            _close(g["topk_actor_logq"][v], want_q[v], 0.0, "top-k log q", abs_tol=tol)

    # Bernoulli mask: exact away from the threshold, either value inside the band
    u = w.uniforms.cpu().numpy()[idx].astype(np.float64)
    band = np.abs(u - o["accept"]) <= MASK_BAND * np.maximum(o["accept"], 1e-30)
    sure = v & ~band
    np.testing.assert_array_equal(g["mask"][sure], o["mask"][sure], err_msg="mask")
    return g, band


def check_batch(buf, w, R, g, flags=0, tol=None):
    """Batch statistics and weights; needs oracle rows for the whole batch."""
    tol = TOL[w.actor.dtype] if tol is None else tol
    mask = np.where(R.out["valid"] == 1, g["mask"], 0).astype(np.int32)     # GPU decision inside the band
    ref = None if w.ref_logprob is None else w.ref_logprob.cpu().numpy().astype(np.float64)
    expected_alpha = bool(flags & obrs.JP_FLAG_ALPHA_EXPECTED)
    b, w_want, rho_want = orc.batch(R.out, mask, w.lam, w.c1, w.c2, ref, expected_alpha)
    st = buf.stats()
    assert st.n_valid == b.n_valid and st.error_flags == 0
    if not expected_alpha:
        assert st.n_accept == b.n_accept
    _close(st.alpha_hat, b.mean_accept if expected_alpha else b.alpha_hat, tol, "alpha_hat")
    _close(st.mean_z_approx, b.mean_z_approx, tol, "mean Z_approx")
    _close(st.kappa, b.kappa, tol, "kappa")
    _close(st.mean_accept, b.mean_accept, tol, "mean a")
    if flags & obrs.JP_FLAG_EXACT_Z:
        _close(st.mean_z_exact, b.mean_z_exact, tol, "mean Z_exact")
    if flags & obrs.JP_FLAG_DISTILL_KL:
        _close(st.mean_distill_kl, b.mean_kl_p_q, tol, "mean KL(p||q)", abs_tol=tol)
    else:
        assert np.isnan(st.mean_distill_kl)
    _close(g["w_obrs"], w_want, tol, "w_OBRS")
    _close(g["rho"], rho_want, tol, "rho")
    return st, b


def check_all(w, flags=0, n_threads=0, tol=None):
    buf = obrs.run_workload(w, flags)
    torch.cuda.synchronize()
    R = run_oracle(w, n_threads)
    g, band = check_rows(buf, w, R, flags=flags, tol=tol)
    st, b = check_batch(buf, w, R, g, flags=flags, tol=tol)
    return buf, R, st
