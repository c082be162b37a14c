"""GPU parity of jp_obrs_forward_stored (actor side as the rollout phase stores it: TopK_inf ids and
log-probabilities plus log p_inf(a_t), Alg. 1 Phase 1) against the float64 oracle, same bars as the
two-tensor form: top-k(p) ids and |V_k| bit-exact, floats within rel 1e-3 (bf16) / 1e-5 (fp32)."""
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
WANT = [n for n in ("accept_prob", "mask", "logq", "logp", "logratio", "z_approx", "w_obrs", "rho",
                    "union_size", "topk_policy", "topk_policy_logp", "stats")]


def _say(msg):
    print(msg, flush=True)


def stored_side(w, k, rows=None):
    """What the rollout phase would have kept of the actor: top-k ids (value desc, id asc) with their
    log-probabilities and the sampled token's log-probability, in float32; computed on the host in
    float64 from the actor logits (harness only)."""
    sel = slice(None) if rows is None else torch.as_tensor(rows, device=w.actor.device)
    a = wl.logits_to_float64(w.actor[sel])
    x = w.sampled_ids[sel].cpu().numpy()
    logq = a - scipy.special.logsumexp(a, axis=1, keepdims=True)
    ids = np.argsort(-a, axis=1, kind="stable")[:, :k].astype(np.int32)
    lq = np.take_along_axis(logq, ids.astype(np.int64), axis=1).astype(np.float32)
    xs = np.clip(x, 0, a.shape[1] - 1)
    lqx = logq[np.arange(a.shape[0]), xs].astype(np.float32)
    return ids, lq, lqx


def run_case(w, rule, flags=0, ids=None, lq=None, lqx=None):
    T, V, k = w.T, w.V, w.k
    if ids is None:
        ids, lq, lqx = stored_side(w, k)
    d_ids = torch.as_tensor(ids, device=DEV)
    d_lq = torch.as_tensor(lq, device=DEV)
    d_lqx = torch.as_tensor(lqx, device=DEV)
    buf = obrs.alloc_buffers(T, V, k, obrs._dtype_code(w.policy), flags, DEV, want=WANT)
    obrs.jp_obrs_forward_stored(w.policy, d_ids, d_lq, d_lqx, w.sampled_ids, w.uniforms, w.ref_logprob,
                                w.lam, k, w.c1, w.c2, flags, rule, buf)
    torch.cuda.synchronize()
    R = orc.rows_stored(wl.logits_to_numpy(w.policy), ids, lq, lqx, w.sampled_ids.cpu().numpy(),
                        w.uniforms.cpu().numpy(), w.lam, k, rule)
    g, band = pu.check_rows(buf, w, R, flags=flags, stored=True)
    st, b = pu.check_batch(buf, w, R, g, flags=flags)
    return buf, R, st


@pytest.mark.parametrize("rule", [0, 1, 2])
def test_tiny_config_fp32(rule):
    _say(f"stored form: tiny fp32 T=64 V=1024 k=32 rule={rule}")
    run_case(wl.tiny(DEV), rule, flags=obrs.JP_FLAG_TOPK_LOGPROBS)


@pytest.mark.parametrize("k,rule", [(1, 1), (16, 2), (64, 1), (64, 0), (128, 2), (256, 1)])
def test_rollout_shape_bf16(k, rule):
    _say(f"stored form: bf16 T=24 V=151936 k={k} rule={rule}")
    w = wl.make_logits(24, wl.QWEN3_VOCAB, torch.bfloat16, seed=wl.BASE_SEED + 3, device=DEV,
                       noise_sigma_range=(0.1, 3.0)).with_params(k=k, lam=1.0)
    run_case(w, rule, flags=obrs.JP_FLAG_TOPK_LOGPROBS)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 37, 255, 515, 4100, 33333])
def test_ragged_shapes_unused_slots_and_repeats(dtype, V):
    k = min(V, 24)
    T = 13
    _say(f"stored form: {dtype} T={T} V={V} k={k}: padded stride, padding rows, unused and repeated slots")
    esz = 2 if dtype == torch.bfloat16 else 4
    stride = (V * esz + 15) // 16 * 16 // esz + 16 // esz * 3
    w = wl.make_logits(T, V, dtype, seed=987 + V, device=DEV, actor_sigma=2.0, spikes=min(3, V),
                       noise_sigma=0.7, pad_every=5, row_stride=stride).with_params(lam=1.3, k=k)
    w.ref_logprob = -torch.rand(T, device=DEV) * 3.0
    ids, lq, lqx = stored_side(w, k)
    ids[1, k // 2] = -1                        # unused slot
    ids[2, k - 1] = ids[2, 0]                  # repeated id: the first occurrence counts
    ids[3, 0] = V + 3                          # outside the vocabulary: unused
    ids[4, :] = -1                             # nothing stored at all
    for rule in (0, 1, 2):
        run_case(w, rule, ids=ids, lq=lq, lqx=lqx)


def test_whole_vocabulary_stored_equals_two_tensor_form():
    _say("stored form: k = V = 256, every rule equals the two-tensor estimate")
    V = 256
    w = wl.make_logits(9, V, torch.float32, seed=77, device=DEV, actor_sigma=2.0, spikes=2,
                       noise_sigma=1.0).with_params(lam=0.8, k=V)
    full = obrs.run_workload(w, 0)
    torch.cuda.synchronize()
    zf = full.z_approx.cpu().numpy()
    for rule in (0, 1, 2):
        buf, R, st = run_case(w, rule)
        np.testing.assert_allclose(buf.z_approx.cpu().numpy(), zf, rtol=2e-5)


def test_rejected_arguments():
    _say("stored form: host-side validation")
    w = wl.tiny(DEV)
    ids, lq, lqx = stored_side(w, w.k)
    d = [torch.as_tensor(a, device=DEV) for a in (ids, lq, lqx)]
    buf = obrs.alloc_buffers(w.T, w.V, w.k, obrs.JP_F32, 0, DEV, want=WANT)

    def call(flags=0, rule=1):
        try:
            obrs.jp_obrs_forward_stored(w.policy, d[0], d[1], d[2], w.sampled_ids, w.uniforms, None, 1.0,
                                        w.k, 3.0, 3.0, flags, rule, buf)
        except obrs.JpError as e:
            return e.status
        return obrs.JP_OK

    assert call() == obrs.JP_OK
    assert call(flags=obrs.JP_FLAG_EXACT_Z) == obrs.JP_ERR_UNSUPPORTED
    assert call(flags=obrs.JP_FLAG_DISTILL_KL) == obrs.JP_ERR_UNSUPPORTED
    assert call(rule=3) == obrs.JP_ERR_PARAM
    torch.cuda.synchronize()


def test_full_size_sampled_rows():
    T, k = 8192, 64
    _say(f"stored form: bf16 T={T} V=151936 k={k} full size, sampled rows")
    w = wl.rollout(DEV, T=T)
    # the stored side is needed for every row: take it from the two-tensor path's own outputs
    # (ids from its top-k list, log-probabilities from its log-prob outputs); the comparison below is
    # against the oracle on the same stored inputs, so their origin does not matter
    full = obrs.run_workload(w, obrs.JP_FLAG_TOPK_LOGPROBS)
    torch.cuda.synchronize()
    d_ids = full.topk_actor.clone()
    d_lq = full.topk_actor_logq.clone()
    d_lqx = full.logq.clone()
    buf = obrs.alloc_buffers(T, w.V, k, obrs.JP_BF16, 0, DEV, want=WANT)
    obrs.jp_obrs_forward_stored(w.policy, d_ids, d_lq, d_lqx, w.sampled_ids, w.uniforms, None, w.lam, k,
                                w.c1, w.c2, 0, obrs.JP_TAIL_KTH, buf)
    torch.cuda.synchronize()
    rows = [0, 1, 63, 64, 1000, 4095, 4096, 8190, 8191]
    sel = torch.as_tensor(rows, device=DEV)
    R = orc.rows_stored(wl.logits_to_numpy(w.policy[sel]), d_ids[sel].cpu().numpy(), d_lq[sel].cpu().numpy(),
                        d_lqx[sel].cpu().numpy(), w.sampled_ids[sel].cpu().numpy(),
                        w.uniforms[sel].cpu().numpy(), w.lam, k, orc.TAIL_KTH)
    pu.check_rows(buf, w, R, rows=rows, stored=True)
    st = buf.stats()
    assert st.n_valid == T and st.error_flags == 0
    # the two estimates bracket: drop <= two-tensor <= k-th bound, row by row
    zk = buf.z_approx.clone()
    obrs.jp_obrs_forward_stored(w.policy, d_ids, d_lq, d_lqx, w.sampled_ids, w.uniforms, None, w.lam, k,
                                w.c1, w.c2, 0, obrs.JP_TAIL_DROP, buf)
    torch.cuda.synchronize()
    zd = buf.z_approx
    zf = full.z_approx
    assert torch.all(zd <= zf * (1 + 2e-3)) and torch.all(zf <= zk * (1 + 2e-3))


@pytest.mark.parametrize("k,rule", [(8, 1), (200, 2)])
def test_bf16_vocabulary_beyond_16_bit_chunk_indices(k, rule):
    """bf16 rows of more than 65 535 16-byte chunks (V > 524 280): the 64-bit chunk descriptors of the
    stored-actor form, with ties, a ragged tail and stored ids past the 16-bit chunk range."""
    V = 524288 + 8 * 21 + 5
    T = 5
    _say(f"stored form: bf16 T={T} V={V} k={k} rule={rule}: 64-bit chunk descriptors")
    w = wl.make_logits(T, V, torch.bfloat16, seed=5151 + k, device=DEV, spikes=4, noise_sigma=1.1,
                       row_stride=(V + 7) // 8 * 8).with_params(lam=1.1, k=k)
    w.policy[1, :] = 0.5                                  # all tied: ids 0..k-1
    w.policy[2, V - 3] = 25.0                             # the ragged tail chunk holds the maximum
    w.actor[3, V - 70000:] += 6.0                         # the stored list lies past the 16-bit chunk range
    w.sampled_ids[3] = V - 1
    buf, R, st = run_case(w, rule, flags=obrs.JP_FLAG_TOPK_LOGPROBS)
    assert buf.topk_policy[1].cpu().tolist() == list(range(k))
    assert int(buf.topk_policy[2, 0]) == V - 3
