"""GPU parity of jp_obrs_forward_lmhead_stored: the target logits come from the matrix cores one
vocabulary chunk at a time (bf16 x bf16 -> fp32, never materialised) and the actor side is what the
rollout phase stored (Alg. 1, Phase 1: TopK_inf ids and log-probabilities, log p_inf(a_t)).

The oracle forms the target logits in float64 from the same bf16 bits and runs its stored-actor
definition on them.  As in the two-head lm_head form the two sides round the logits differently
(~1e-5), so top-k(p) may differ where two logits are nearly tied: a list is accepted if, rank by
rank, the float64 logit of the GPU's id is within 1e-4 max(1, |l|) of the oracle's, and Z_approx is
then compared on the set the GPU chose.  Floats: the bf16-input bar (rel 1e-3, absolute for
log-domain values)."""
import numpy as np
import pytest
import scipy.special
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from oracle import obrs_oracle as orc
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl
    import parity_util as pu

DEV = "cuda"
TOL = 1e-3
MASK_BAND = 1e-4      # fp32-accumulated logits: a(x) carries a few 1e-5 of relative rounding
TIE = 1e-4
WANT = ["accept_prob", "mask", "logq", "logp", "logratio", "z_approx", "w_obrs", "rho", "union_size",
        "topk_policy", "topk_policy_logp", "stats"]


def _say(msg):
    print(msg, flush=True)


def stored_side(w, k, rows):
    """What the rollout phase would have kept of the actor head's distribution (harness only):
    float64 on the host from the actor head's hidden states and weights."""
    r = torch.as_tensor(rows, device=DEV)
    a = orc.lm_head_logits(wl.logits_to_numpy(w.H_actor[r]), wl.logits_to_numpy(w.W_actor))
    logq = a - scipy.special.logsumexp(a, axis=1, keepdims=True)
    ids = np.argsort(-a, axis=1, kind="stable")[:, :k].astype(np.int32)
    lq = np.take_along_axis(logq, ids.astype(np.int64), axis=1).astype(np.float32)
    x = w.sampled_ids.cpu().numpy()[rows]
    lqx = logq[np.arange(len(rows)), np.clip(x, 0, a.shape[1] - 1)].astype(np.float32)
    return ids, lq, lqx


def z_on_set(lp, lse_p, ids, lq, topk_p, lam, rule, V):
    """Z_approx of the stored form on a given top-k(p) set, from its definition (used only for rows
    where a near-tie made the GPU's list differ from the oracle's)."""
    stored = {}
    for j, v in enumerate(ids.tolist()):
        if 0 <= v < V and v not in stored:
            stored[v] = float(lq[j])
    n = len(stored)
    kth = min(stored.values()) if n else 0.0
    if rule == 0 or n == V:
        tail = -np.inf
    elif rule == 1:
        tail = kth
    else:
        rest = max(1.0 - sum(np.exp(v) for v in stored.values()), 0.0)
        with np.errstate(divide="ignore"):
            tail = min(float(np.log(rest / (V - n))), kth)
    z = sum(min(np.exp(q), np.exp(lp[v] - lse_p) / lam) for v, q in stored.items())
    extra = [v for v in topk_p.tolist() if v not in stored]
    z += sum(min(np.exp(tail), np.exp(lp[v] - lse_p) / lam) for v in extra)
    return z, n + len(extra)


def run_case(w, rule, rows, flags=0, vocab_chunk=0, stored=None, batch=True):
    T, V, k = w.T, w.V, w.k
    ids, lq, lqx = stored if stored is not None else stored_side(w, k, np.arange(T))
    d_ids, d_lq, d_lqx = (torch.as_tensor(a, device=DEV) for a in (ids, lq, lqx))
    d_p = w.H_policy.shape[1]
    nbytes = obrs.jp_obrs_lmhead_stored_workspace_bytes(T, V, d_p, k, vocab_chunk)
    assert nbytes > 0
    buf = obrs.alloc_buffers(T, V, k, obrs.JP_F32, flags, DEV, want=WANT, workspace_bytes=nbytes)
    obrs.jp_obrs_forward_lmhead_stored(w.H_policy, w.W_policy, d_ids, d_lq, d_lqx, w.sampled_ids, w.uniforms,
                                       w.ref_logprob, w.lam, k, w.c1, w.c2, flags, rule, buf, vocab_chunk)
    torch.cuda.synchronize()

    r = torch.as_tensor(rows, device=DEV)
    lp = orc.lm_head_logits(wl.logits_to_numpy(w.H_policy[r]), wl.logits_to_numpy(w.W_policy))
    x = w.sampled_ids.cpu().numpy()[rows]
    u = w.uniforms.cpu().numpy()[rows]
    R = orc.rows_stored(lp, ids[rows], lq[rows], lqx[rows], x, u, w.lam, k, rule)
    o = R.out
    valid = o["valid"] == 1
    g = {n: t.cpu().numpy()[rows] for n, t in buf.tensors.items() if n != "stats"}
    v = valid
    if (~v).any():
        for n in ("accept_prob", "logq", "logp", "logratio", "z_approx"):
            assert np.all(g[n][~v] == 0.0), n
        assert np.all(g["mask"][~v] == 0) and np.all(g["topk_policy"][~v] == -1)
    pu._close(g["logq"][v], o["logq_x"][v], 0.0, "log q(x)", abs_tol=TOL)
    pu._close(g["logp"][v], o["logp_x"][v], 0.0, "log p(x)", abs_tol=TOL)
    pu._close(g["logratio"][v], o["logratio"][v], 0.0, "log ratio", abs_tol=TOL)
    pu._close(g["accept_prob"][v], o["accept"][v], TOL, "a(x)")
    n_swapped = 0
    z_ref = o["z_approx"].copy()
    for i in np.nonzero(v)[0]:
        got, want, l = g["topk_policy"][i], R.topk_p[i], lp[i]
        assert len(set(got.tolist())) == k and got.min() >= 0 and got.max() < V
        if np.array_equal(got, want):
            assert g["union_size"][i] == o["union_size"][i]
        else:
            n_swapped += 1
            d = np.abs(l[got] - l[want])
            assert np.all(d <= TIE * np.maximum(1.0, np.abs(l[want]))), (rows[i], d.max())
            z_ref[i], usize = z_on_set(l, o["lse_p"][i], ids[rows[i]], lq[rows[i]], got, w.lam, rule, V)
            assert g["union_size"][i] == usize
        pu._close(g["z_approx"][i], z_ref[i], TOL, "Z_approx")
        if flags & obrs.JP_FLAG_TOPK_LOGPROBS:
            pu._close(g["topk_policy_logp"][i], l[got] - o["lse_p"][i], 0.0, "top-k log p", abs_tol=TOL)
    band = np.abs(u - o["accept"]) <= MASK_BAND * np.maximum(o["accept"], 1e-30)
    np.testing.assert_array_equal(g["mask"][v & ~band], o["mask"][v & ~band])
    if batch:                                              # rows == all rows
        rows_for_batch = o.copy()
        rows_for_batch["z_approx"] = z_ref
        mask = np.where(v, g["mask"], 0).astype(np.int32)
        ref = None if w.ref_logprob is None else w.ref_logprob.cpu().numpy().astype(np.float64)
        b, w_want, rho_want = orc.batch(rows_for_batch, mask, w.lam, w.c1, w.c2, ref)
        st = buf.stats()
        assert st.n_valid == b.n_valid and st.n_accept == b.n_accept and st.error_flags == 0
        pu._close(st.kappa, b.kappa, TOL, "kappa")
        pu._close(g["w_obrs"][v], w_want[v], TOL, "w_OBRS")
        pu._close(g["rho"][v], rho_want[v], TOL, "rho")
    return buf, n_swapped


@pytest.mark.parametrize("rule", [0, 1, 2])
@pytest.mark.parametrize("T,V,da,dp,k,chunk", [
    (48, 3000, 128, 192, 16, 512),       # several chunk groups, ragged last chunk, ragged row tile
    (300, 1000, 64, 64, 8, 256),         # more than one row tile
    (17, 700, 64, 128, 64, 0),           # single chunk
    (33, 5000, 256, 128, 100, 1024),     # k class 128
    (9, 2600, 64, 64, 200, 512),         # k class 256
])
def test_small_shapes(T, V, da, dp, k, chunk, rule):
    _say(f"lm_head + stored actor: T={T} V={V} d_policy={dp} k={k} chunk={chunk} rule={rule}")
    w = wl.lm_head(T, V, da, dp, DEV, seed=300 + T, k=k).with_params(lam=1.2)
    w.ref_logprob = -torch.rand(T, device=DEV)
    run_case(w, rule, np.arange(T), flags=obrs.JP_FLAG_TOPK_LOGPROBS, vocab_chunk=chunk)


def test_padding_rows_unused_and_repeated_slots():
    T, V, k = 21, 1500, 12
    _say(f"lm_head + stored actor: T={T} V={V} k={k}: padding rows, unused and repeated slots")
    w = wl.lm_head(T, V, 64, 128, DEV, seed=41, k=k).with_params(lam=0.9)
    w.sampled_ids[5] = -1
    w.sampled_ids[11] = -7
    ids, lq, lqx = stored_side(w, k, np.arange(T))
    ids[1, k // 2] = -1                        # unused slot
    ids[2, k - 1] = ids[2, 0]                  # repeated id: the first occurrence counts
    ids[3, 0] = V + 3                          # outside the vocabulary: unused
    ids[4, :] = -1                             # nothing stored at all
    for rule in (0, 1, 2):
        run_case(w, rule, np.arange(T), vocab_chunk=256, stored=(ids, lq, lqx))


def test_matches_the_materialised_stored_form():
    """Same inputs through jp_obrs_forward_stored on fp32 logits made by torch: ids agree except at
    near-ties and the scalars agree to the bf16 bar."""
    _say("lm_head + stored actor vs materialised fp32 target logits, T=64 V=20000")
    w = wl.lm_head(64, 20000, 128, 256, DEV, seed=8, k=32)
    stored = stored_side(w, w.k, np.arange(w.T))
    buf, _ = run_case(w, obrs.JP_TAIL_KTH, np.arange(w.T), vocab_chunk=2048, stored=stored)
    lp = (w.H_policy.float() @ w.W_policy.float()).contiguous()
    bm = obrs.alloc_buffers(w.T, w.V, w.k, obrs.JP_F32, 0, DEV, want=WANT)
    d = [torch.as_tensor(a, device=DEV) for a in stored]
    obrs.jp_obrs_forward_stored(lp, d[0], d[1], d[2], w.sampled_ids, w.uniforms, None, w.lam, w.k, w.c1, w.c2,
                                0, obrs.JP_TAIL_KTH, bm)
    torch.cuda.synchronize()
    same = (buf.topk_policy == bm.topk_policy).all(dim=1)
    assert same.float().mean() > 0.9
    np.testing.assert_allclose(buf.z_approx[same].cpu().numpy(), bm.z_approx[same].cpu().numpy(), rtol=1e-4)
    np.testing.assert_allclose(buf.logratio.cpu().numpy(), bm.logratio.cpu().numpy(), atol=1e-4)


def test_vocab_major_weights_give_the_same_bits():
    _say("lm_head + stored actor: [V, d] weights")
    w = wl.lm_head(48, 3000, 128, 192, DEV, seed=51, k=16)
    stored = stored_side(w, w.k, np.arange(w.T))
    ref, _ = run_case(w, obrs.JP_TAIL_REST, np.arange(w.T), vocab_chunk=512, stored=stored)
    wt = w.with_params(W_policy=w.W_policy.t().contiguous())
    d = [torch.as_tensor(a, device=DEV) for a in stored]
    nbytes = obrs.jp_obrs_lmhead_stored_workspace_bytes(w.T, w.V, 192, w.k, 512)
    got = obrs.alloc_buffers(w.T, w.V, w.k, obrs.JP_F32, 0, DEV, want=WANT, workspace_bytes=nbytes)
    obrs.jp_obrs_forward_lmhead_stored(wt.H_policy, wt.W_policy, d[0], d[1], d[2], w.sampled_ids, w.uniforms,
                                       w.ref_logprob, w.lam, w.k, w.c1, w.c2, obrs.JP_FLAG_W_VOCAB_MAJOR,
                                       obrs.JP_TAIL_REST, got, 512)
    torch.cuda.synchronize()
    for n in ref.tensors:
        assert n == "stats" or torch.equal(got.tensors[n], ref.tensors[n]), n
    assert got.stats().kappa == ref.stats().kappa


def test_can_be_captured_in_a_hip_graph():
    _say("lm_head + stored actor: T=48 V=3000 captured in a graph, replayed three times with eager work between")
    w = wl.lm_head(48, 3000, 128, 192, DEV, seed=61, k=16)
    stored = stored_side(w, w.k, np.arange(w.T))
    d = [torch.as_tensor(a, device=DEV) for a in stored]
    nbytes = obrs.jp_obrs_lmhead_stored_workspace_bytes(w.T, w.V, 192, w.k, 512)
    buf = obrs.alloc_buffers(w.T, w.V, w.k, obrs.JP_F32, 0, DEV, want=WANT, workspace_bytes=nbytes)

    def step():
        obrs.jp_obrs_forward_lmhead_stored(w.H_policy, w.W_policy, d[0], d[1], d[2], w.sampled_ids, w.uniforms,
                                           None, w.lam, w.k, w.c1, w.c2, 0, obrs.JP_TAIL_KTH, buf, 512)

    step()
    torch.cuda.synchronize()
    ref = {n: t.clone() for n, t in buf.tensors.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                            # warm-up on the capture side
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in buf.tensors.values():
            t.zero_()                                     # eager work between the replays
        buf.workspace.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in ref:
            same = torch.equal(buf.tensors[n], ref[n]) or (
                ref[n].is_floating_point() and torch.equal(torch.nan_to_num(buf.tensors[n]), torch.nan_to_num(ref[n])))
            assert same, (rep, n)


def test_rejected_arguments():
    _say("lm_head + stored actor: host-side validation")
    w = wl.lm_head(8, 512, 64, 64, DEV, seed=3, k=4)
    stored = stored_side(w, 4, np.arange(8))
    d = [torch.as_tensor(a, device=DEV) for a in stored]
    nbytes = obrs.jp_obrs_lmhead_stored_workspace_bytes(8, 512, 64, 4, 0)
    buf = obrs.alloc_buffers(8, 512, 4, obrs.JP_F32, 0, DEV, want=WANT, workspace_bytes=nbytes)

    def call(flags=0, rule=1, b=buf):
        try:
            obrs.jp_obrs_forward_lmhead_stored(w.H_policy, w.W_policy, d[0], d[1], d[2], w.sampled_ids,
                                               w.uniforms, None, 1.0, 4, 3.0, 3.0, flags, rule, b)
        except obrs.JpError as e:
            return e.status
        return obrs.JP_OK

    assert call() == obrs.JP_OK
    assert call(flags=obrs.JP_FLAG_EXACT_Z) == obrs.JP_ERR_UNSUPPORTED
    assert call(flags=obrs.JP_FLAG_DISTILL_KL) == obrs.JP_ERR_UNSUPPORTED
    assert call(rule=3) == obrs.JP_ERR_PARAM
    small = obrs.alloc_buffers(8, 512, 4, obrs.JP_F32, 0, DEV, want=WANT)
    assert call(b=small) == obrs.JP_ERR_WORKSPACE
    assert obrs.jp_obrs_lmhead_stored_workspace_bytes(8, 512, 60, 4, 0) == 0      # d not a multiple of 64
    torch.cuda.synchronize()


def test_full_size_sampled_rows():
    """T=16384, d=4096, V=151936, k=64: sampled rows against the oracle, batch statistics through
    their defining relations on the per-row outputs."""
    _say("lm_head + stored actor, full size: T=16384 V=151936 d_policy=4096 k=64")
    w = wl.lm_head(device=DEV)
    T, k = w.T, w.k
    rng = np.random.default_rng(20260211)
    rows = np.unique(np.concatenate([[0, 1, T - 2, T - 1], rng.integers(0, T, 256)]))
    # The stored side is needed for every row: an arbitrary but valid one (ids spread over the
    # vocabulary, log-probabilities of a geometric tail) except on the sampled rows, which get the
    # actor head's true top-k.  The comparison is against the oracle on the same stored inputs.
    gen = torch.Generator(device="cpu").manual_seed(77)
    ids = torch.stack([torch.randperm(w.V, generator=gen)[:k] for _ in range(64)]).to(torch.int32)
    ids = ids.repeat(T // 64, 1).numpy().copy()
    lq = np.tile((-3.0 - 0.1 * np.arange(k, dtype=np.float32))[None, :], (T, 1))
    lqx = np.full(T, -4.0, dtype=np.float32)
    s_ids, s_lq, s_lqx = stored_side(w, k, rows)
    ids[rows], lq[rows], lqx[rows] = s_ids, s_lq, s_lqx
    buf, n_swapped = run_case(w, obrs.JP_TAIL_KTH, rows, stored=(ids, lq, lqx), batch=False)
    _say(f"  lists with a near-tie swap among {len(rows)}: {n_swapped}")
    st = buf.stats()
    g = {n: buf.tensors[n].cpu().numpy().astype(np.float64) for n in ("z_approx", "logratio", "w_obrs", "mask")}
    assert st.error_flags == 0 and st.n_valid == T and st.n_accept == int(g["mask"].sum())
    assert st.kappa == pytest.approx(g["mask"].mean() / g["z_approx"].mean(), rel=1e-9)
    np.testing.assert_allclose(g["w_obrs"], st.kappa * g["z_approx"] * np.maximum(w.lam, np.exp(g["logratio"])), rtol=1e-5)
