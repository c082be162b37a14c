"""GPU parity of the fused lm_head form: logits come from the matrix cores (bf16 x bf16 -> fp32)
one vocabulary chunk at a time; the oracle forms them in float64 from the same bf16 bits.

Because the two sides round the logits differently (~1e-5), a top-k list may differ from the
oracle's where two logits are nearly tied: an id list is accepted if, rank by rank, the float64
logit of the GPU's id is within 1e-4 max(1, |l|) of the oracle's; Z_approx is then compared on the
set the GPU chose.  Floats: the bf16-input bar (rel 1e-3, absolute for log-domain values).  The
Bernoulli draw: a logit accumulated in fp32 over d products carries ~1e-5 of rounding, so a(x)
differs from the oracle's by a few 1e-5 relative and a uniform within 1e-4 a of it may fall on
either side (the materialised path's band is 1e-5 because its logits are exact inputs)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from oracle import obrs_oracle as orc
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl
    import parity_util as pu

DEV = "cuda"
TOL = 1e-3
TIE = 1e-4
MASK_BAND = 1e-4


def _run(w, flags=0, vocab_chunk=0):
    T = w.T
    V = w.W_actor.shape[0] if flags & obrs.JP_FLAG_W_VOCAB_MAJOR else w.V
    nbytes = obrs.jp_obrs_lmhead_workspace_bytes(T, V, w.H_actor.shape[1], w.H_policy.shape[1], w.k, vocab_chunk)
    assert nbytes > 0
    buf = obrs.alloc_buffers(T, V, w.k, obrs.JP_F32, flags, DEV, workspace_bytes=nbytes)
    obrs.jp_obrs_forward_lmhead(w.H_actor, w.W_actor, w.H_policy, w.W_policy, w.sampled_ids, w.uniforms,
                                w.ref_logprob, w.lam, w.k, w.c1, w.c2, flags, buf, vocab_chunk)
    torch.cuda.synchronize()
    return buf


def _check(w, buf, rows, flags=0, batch=True):
    r = torch.as_tensor(rows, device=w.H_actor.device)
    lq = orc.lm_head_logits(wl.logits_to_numpy(w.H_actor[r]), wl.logits_to_numpy(w.W_actor))
    lp = orc.lm_head_logits(wl.logits_to_numpy(w.H_policy[r]), wl.logits_to_numpy(w.W_policy))
    x = w.sampled_ids.cpu().numpy()[rows]
    u = w.uniforms.cpu().numpy()[rows]
    R = orc.rows(lq, lp, x, u, w.lam, w.k)
    o = R.out
    g = {n: t.cpu().numpy()[rows] for n, t in buf.tensors.items() if n != "stats"}
    pu._close(g["logq"], o["logq_x"], 0.0, "log q(x)", abs_tol=TOL)
    pu._close(g["logp"], o["logp_x"], 0.0, "log p(x)", abs_tol=TOL)
    pu._close(g["logratio"], o["logratio"], 0.0, "log ratio", abs_tol=TOL)
    pu._close(g["accept_prob"], o["accept"], TOL, "a(x)")
    if flags & obrs.JP_FLAG_DISTILL_KL:
        pu._close(g["distill_kl"], o["kl_p_q"], TOL, "KL(p||q)", abs_tol=TOL)
    n_swapped = 0
    for i in range(len(rows)):
        for got, want, l in ((g["topk_actor"][i], R.topk_q[i], lq[i]), (g["topk_policy"][i], R.topk_p[i], lp[i])):
            assert len(set(got.tolist())) == w.k and got.min() >= 0 and got.max() < w.V
            if not np.array_equal(got, want):
                n_swapped += 1
                d = np.abs(l[got] - l[want])
                assert np.all(d <= TIE * np.maximum(1.0, np.abs(l[want]))), (rows[i], d.max())
        logq = lq[i] - o["lse_q"][i]
        logp = lp[i] - o["lse_p"][i]
        U = np.array(sorted(set(g["topk_actor"][i].tolist()) | set(g["topk_policy"][i].tolist())))
        assert g["union_size"][i] == len(U)
        z = np.minimum(np.exp(logq[U]), np.exp(logp[U]) / w.lam).sum()
        pu._close(g["z_approx"][i], z, TOL, "Z_approx on the GPU's set")
        if np.array_equal(g["topk_actor"][i], R.topk_q[i]) and np.array_equal(g["topk_policy"][i], R.topk_p[i]):
            pu._close(g["z_approx"][i], o["z_approx"][i], TOL, "Z_approx")
        if flags & obrs.JP_FLAG_TOPK_LOGPROBS:
            pu._close(g["topk_actor_logq"][i], logq[g["topk_actor"][i]], 0.0, "top-k log q", abs_tol=TOL)
            pu._close(g["topk_policy_logp"][i], logp[g["topk_policy"][i]], 0.0, "top-k log p", abs_tol=TOL)
    band = np.abs(u - o["accept"]) <= MASK_BAND * np.maximum(o["accept"], 1e-30)
    np.testing.assert_array_equal(g["mask"][~band], o["mask"][~band])
    if batch:      # rows == all rows
        mask = g["mask"].astype(np.int32)
        rows_for_batch = o.copy()
        rows_for_batch["z_approx"] = g["z_approx"]          # GPU's sets where near-ties swapped
        b, w_want, rho_want = orc.batch(rows_for_batch, mask, w.lam, w.c1, w.c2,
                                        None if w.ref_logprob is None else w.ref_logprob.cpu().numpy().astype(np.float64))
        st = buf.stats()
        assert st.n_valid == b.n_valid and st.n_accept == b.n_accept and st.error_flags == 0
        pu._close(st.kappa, b.kappa, TOL, "kappa")
        pu._close(g["w_obrs"], w_want, TOL, "w_OBRS")
        pu._close(g["rho"], rho_want, TOL, "rho")
    return n_swapped


@pytest.mark.parametrize("T,V,da,dp,k,chunk", [
    (48, 3000, 128, 192, 16, 512),       # several chunks, ragged last chunk, ragged row tile
    (300, 1000, 64, 64, 8, 256),         # more than one row tile
    (17, 700, 64, 128, 64, 0),           # single chunk
    (33, 5000, 256, 128, 100, 1024),     # k class 128
])
def test_lmhead_small_shapes(T, V, da, dp, k, chunk):
    print(f"lm_head T={T} V={V} d=({da},{dp}) k={k} chunk={chunk}", flush=True)
    w = wl.lm_head(T, V, da, dp, DEV, seed=100 + T, k=k).with_params(lam=1.2)
    w.ref_logprob = -torch.rand(T, device=DEV)
    flags = obrs.JP_FLAG_TOPK_LOGPROBS | obrs.JP_FLAG_DISTILL_KL
    buf = _run(w, flags, chunk)
    _check(w, buf, np.arange(T), flags)


@pytest.mark.parametrize("T,V,da,dp,k,chunk", [
    (48, 3000, 128, 192, 16, 512),       # full chunks used in place, the ragged last one copied and padded
    (17, 700, 64, 128, 64, 0),           # single, partial chunk
    (40, 2048, 64, 64, 32, 1024),        # V a multiple of the chunk: nothing is copied
])
def test_lmhead_vocab_major_weights_give_the_same_bits(T, V, da, dp, k, chunk):
    print(f"lm_head [V, d] weights T={T} V={V} d=({da},{dp}) k={k} chunk={chunk}", flush=True)
    w = wl.lm_head(T, V, da, dp, DEV, seed=200 + T, k=k)
    flags = obrs.JP_FLAG_TOPK_LOGPROBS
    ref = _run(w, flags, chunk)
    wt = w.with_params(W_actor=w.W_actor.t().contiguous(), W_policy=w.W_policy.t().contiguous())
    got = _run(wt, flags | obrs.JP_FLAG_W_VOCAB_MAJOR, chunk)
    for n in ref.tensors:
        assert torch.equal(got.tensors[n], ref.tensors[n]) or n == "stats", n
    assert got.stats().kappa == ref.stats().kappa


def test_lmhead_matches_materialised_path():
    """Same inputs through jp_obrs_forward on fp32 logits made by torch: ids agree except at
    near-ties and the scalars agree to the bf16 bar."""
    print("lm_head vs materialised fp32 logits, T=64 V=20000", flush=True)
    w = wl.lm_head(64, 20000, 128, 256, DEV, seed=7, k=32)
    buf = _run(w, 0, 2048)
    la = (w.H_actor.float() @ w.W_actor.float()).contiguous()
    lp = (w.H_policy.float() @ w.W_policy.float()).contiguous()
    wm = wl.Workload("mat", la, lp, w.sampled_ids, w.uniforms, lam=w.lam, k=w.k)
    bm = obrs.run_workload(wm)
    torch.cuda.synchronize()
    same = (buf.topk_actor == bm.topk_actor).all(dim=1) & (buf.topk_policy == bm.topk_policy).all(dim=1)
    assert same.float().mean() > 0.9
    np.testing.assert_allclose(buf.z_approx[same].cpu().numpy(), bm.z_approx[same].cpu().numpy(), rtol=1e-4)
    np.testing.assert_allclose(buf.logratio.cpu().numpy(), bm.logratio.cpu().numpy(), atol=1e-4)


def test_lmhead_rejects_bad_arguments():
    w = wl.lm_head(8, 512, 64, 64, DEV, seed=3, k=4)
    buf = obrs.alloc_buffers(8, 512, 4, obrs.JP_F32, 0, DEV, workspace_bytes=obrs.jp_obrs_lmhead_workspace_bytes(8, 512, 64, 64, 4, 0))
    with pytest.raises(obrs.JpError) as e:
        obrs.jp_obrs_forward_lmhead(w.H_actor, w.W_actor, w.H_policy, w.W_policy, w.sampled_ids, w.uniforms,
                                    None, 1.0, 4, 3.0, 3.0, obrs.JP_FLAG_EXACT_Z, buf)
    assert e.value.status == obrs.JP_ERR_UNSUPPORTED
    assert obrs.jp_obrs_lmhead_workspace_bytes(8, 512, 60, 64, 4, 0) == 0      # d not a multiple of 64
    small = obrs.alloc_buffers(8, 512, 4, obrs.JP_F32, 0, DEV)
    with pytest.raises(obrs.JpError) as e:
        obrs.jp_obrs_forward_lmhead(w.H_actor, w.W_actor, w.H_policy, w.W_policy, w.sampled_ids, w.uniforms,
                                    None, 1.0, 4, 3.0, 3.0, 0, small)
    assert e.value.status == obrs.JP_ERR_WORKSPACE


def _materialised_fp32(w):
    """The same logits through an independent fp32 GEMM of the harness (torch.mm on the widened bf16
    values, row blocks), then the materialised two-tensor path on them."""
    T, V = w.T, w.V
    la = torch.empty((T, V), dtype=torch.float32, device=DEV)
    lp = torch.empty((T, V), dtype=torch.float32, device=DEV)
    Wa, Wp = w.W_actor.float(), w.W_policy.float()
    for r0 in range(0, T, 2048):
        torch.mm(w.H_actor[r0:r0 + 2048].float(), Wa, out=la[r0:r0 + 2048])
        torch.mm(w.H_policy[r0:r0 + 2048].float(), Wp, out=lp[r0:r0 + 2048])
    del Wa, Wp
    wm = wl.Workload("materialised", la, lp, w.sampled_ids, w.uniforms, lam=w.lam, k=w.k, c1=w.c1, c2=w.c2)
    bm = obrs.run_workload(wm)
    torch.cuda.synchronize()
    return bm


def test_lmhead_full_size():
    """T=16384, d=2048/4096, V=151936, k=64.  256 seeded rows (and the first and last) against the
    oracle on float64 logits; the batch stage (Sec. 4.4.2, Alg. 1 step 3), which needs every row,
    against the materialised path run on logits from an independent fp32 GEMM of the harness (that
    path is compared with the oracle over whole batches elsewhere)."""
    print("lm_head full size: T=16384 V=151936 d=(2048,4096) k=64", flush=True)
    w = wl.lm_head(device=DEV)
    buf = _run(w, 0, 0)
    rng = np.random.default_rng(20260210)
    rows = np.unique(np.concatenate([[0, 1, w.T - 2, w.T - 1], rng.integers(0, w.T, 256)]))
    assert len(rows) >= 256
    n_swapped = _check(w, buf, rows, 0, batch=False)
    print(f"  {len(rows)} rows against the oracle; lists with a near-tie swap among {2 * len(rows)}: {n_swapped}", flush=True)

    bm = _materialised_fp32(w)
    st, sm = buf.stats(), bm.stats()
    g = {n: buf.tensors[n].cpu().numpy().astype(np.float64) for n in buf.tensors if n != "stats"}
    m = {n: bm.tensors[n].cpu().numpy().astype(np.float64) for n in bm.tensors if n != "stats"}
    assert st.error_flags == 0 and sm.error_flags == 0 and st.n_valid == w.T == sm.n_valid
    u = w.uniforms.cpu().numpy().astype(np.float64)
    band = np.abs(u - m["accept_prob"]) <= MASK_BAND * np.maximum(m["accept_prob"], 1e-30)
    np.testing.assert_array_equal(g["mask"][~band], m["mask"][~band])
    assert abs(st.n_accept - sm.n_accept) <= int(band.sum())
    pu._close(g["logq"], m["logq"], 0.0, "log q(x) vs materialised", abs_tol=TOL)
    pu._close(g["logp"], m["logp"], 0.0, "log p(x) vs materialised", abs_tol=TOL)
    pu._close(g["accept_prob"], m["accept_prob"], TOL, "a(x) vs materialised")
    same = (g["topk_actor"] == m["topk_actor"]).all(axis=1) & (g["topk_policy"] == m["topk_policy"]).all(axis=1)
    print(f"  rows whose two id lists equal the materialised path's: {int(same.sum())} of {w.T}", flush=True)
    assert same.mean() > 0.9
    # A near-tie swap exchanges two tokens of almost equal logit under one model at the k-th place of
    # its list; their terms min(q, p/lambda) may differ by up to that k-th probability, about
    # Z_approx / k on these flat rows.  Per-row values are compared where the lists agree, batch
    # means with that allowance for the rows where they do not.
    slack = TOL + (1.0 - same.mean()) * 2.0 / w.k
    pu._close(g["z_approx"][same], m["z_approx"][same], TOL, "Z_approx vs materialised")
    pu._close(st.mean_z_approx, sm.mean_z_approx, slack, "mean Z_approx vs materialised")
    pu._close(st.mean_accept, sm.mean_accept, TOL, "mean a vs materialised")
    adj = sm.alpha_hat / st.alpha_hat            # 1 unless a uniform inside the band fell on the other side
    pu._close(st.kappa * adj, sm.kappa, slack, "kappa vs materialised")
    pu._close(g["w_obrs"][same] * adj, m["w_obrs"][same], slack, "w_OBRS vs materialised")
    # the batch stage's own relations on the per-row outputs
    assert st.n_accept == int(g["mask"].sum())
    assert st.kappa == pytest.approx(g["mask"].mean() / g["z_approx"].mean(), rel=1e-9)
    np.testing.assert_allclose(g["w_obrs"], st.kappa * g["z_approx"] * np.maximum(w.lam, np.exp(g["logratio"])), rtol=1e-5)
    np.testing.assert_allclose(g["rho"], np.minimum(g["w_obrs"], w.c1), rtol=1e-6)
    print(f"  alpha_hat={st.alpha_hat:.4f} mean Z_approx={st.mean_z_approx:.4f} kappa={st.kappa:.4f} "
          f"(materialised fp32 path: {sm.alpha_hat:.4f} {sm.mean_z_approx:.4f} {sm.kappa:.4f})", flush=True)
