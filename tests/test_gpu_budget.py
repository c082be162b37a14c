"""GPU parity of jp_obrs_lambda_for_budget (Sec. 3.3, Theorem 2: the scaling factor that meets an
acceptance budget) against the float64 oracle, which finds it exactly by sorting the ratios."""
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


def _say(msg):
    print(msg, flush=True)


def _check(w, target, row_target=None, rows=None):
    """Two bars.  (1) The budget is met: Z(lambda_gpu) = abar within the float tolerance, with Z
    recomputed here in float64.  (2) lambda itself matches the oracle's within tolerance x condition
    number of the problem, cond = abar / (abar - A) with A the q-mass above lambda (d lambda / lambda =
    -cond d abar / abar): near abar = 1 the p-side mass abar - A vanishes and lambda is not determined
    to any useful precision by the budget, so only bar (1) applies there."""
    buf = obrs.run_workload(w, 0)
    rt = None if row_target is None else torch.as_tensor(row_target, dtype=torch.float32, device=DEV)
    lam = obrs.jp_obrs_lambda_for_budget(w.actor, w.policy, target, buf, row_target=rt)
    torch.cuda.synchronize()
    idx = np.arange(w.T) if rows is None else np.asarray(rows)
    sel = torch.as_tensor(idx, device=DEV)
    x = w.sampled_ids[sel].cpu().numpy()
    rt_np = None if row_target is None else np.asarray(row_target, dtype=np.float32)[idx]
    want = orc.lambda_for_budget_rows(wl.logits_to_numpy(w.actor[sel]), wl.logits_to_numpy(w.policy[sel]),
                                      x, target, rt_np)
    got = lam[sel].cpu().numpy().astype(np.float64)
    tol = pu.TOL[w.actor.dtype]
    bad_budget = np.zeros(len(idx), dtype=bool) if rt_np is None else ~((rt_np > 0) & (rt_np <= 1))
    assert np.all(got[x < 0] == 0.0)
    assert np.all(np.isnan(got[(x >= 0) & bad_budget])) and np.all(np.isnan(want[(x >= 0) & bad_budget]))
    a64 = wl.logits_to_float64(w.actor[sel])
    p64 = wl.logits_to_float64(w.policy[sel])
    import scipy.special
    n_lambda = 0
    for i in range(len(idx)):
        if x[i] < 0 or bad_budget[i]:
            continue
        abar = float(target if rt_np is None else rt_np[i])
        q, p = scipy.special.softmax(a64[i]), scipy.special.softmax(p64[i])
        zmax = float(q[p > 0].sum())
        z_got = float(np.minimum(q, p / got[i]).sum())
        assert abs(z_got - min(abar, zmax)) <= tol * abar, (idx[i], abar, z_got, got[i], want[i])
        with np.errstate(divide="ignore", invalid="ignore"):
            A = float(q[(p / q > want[i]) & (p > 0)].sum())
        cond = abar / max(abar - A, 1e-300)
        if cond <= 100.0:
            n_lambda += 1
            assert abs(got[i] - want[i]) <= tol * (1.0 + cond) * want[i], (idx[i], abar, got[i], want[i], cond)
    return lam, n_lambda


@pytest.mark.parametrize("target", [1.0, 0.97, 0.5, 0.1, 1e-3])
def test_tiny_config_fp32(target):
    _say(f"budget: tiny fp32 T=64 V=1024 abar={target}")
    _check(wl.tiny(DEV), target)


def test_rollout_shape_bf16_per_row_budgets():
    _say("budget: bf16 T=24 V=151936, per-row budgets, two of them invalid")
    w = wl.make_logits(24, wl.QWEN3_VOCAB, torch.bfloat16, seed=wl.BASE_SEED + 3, device=DEV,
                       noise_sigma_range=(0.1, 3.0)).with_params(k=8)
    rt = np.concatenate([np.linspace(0.02, 1.0, 22), [0.0, 1.5]]).astype(np.float32)
    _check(w, 0.5, row_target=rt)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 37, 255, 515, 4100, 33333])
def test_ragged_shapes_and_masked_entries(dtype, V):
    T = 13
    _say(f"budget: {dtype} T={T} V={V}, padded stride, padding rows, -inf entries")
    esz = 2 if dtype == torch.bfloat16 else 4
    stride = (V * esz + 15) // 16 * 16 // esz + 16 // esz * 3
    w = wl.make_logits(T, V, dtype, seed=246 + V, device=DEV, actor_sigma=2.0, spikes=min(3, V),
                       noise_sigma=0.7, pad_every=5, row_stride=stride).with_params(k=min(V, 8))
    w.actor[3, : V // 3] = float("-inf")
    w.policy[3, V // 2:] = float("-inf")
    w.sampled_ids[3] = V // 3 + 1 if V // 3 + 1 < V // 2 else V // 3      # a token both models can emit
    for target in (1.0, 0.6, 0.05):
        _check(w, target)


def test_matched_distributions_closed_form():
    _say("budget: p == q -> lambda = 1 / abar")
    w = wl.make_logits(6, 5000, torch.float32, seed=8, device=DEV)
    w = w.with_params(policy=w.actor.clone(), k=8)
    rt = np.array([1.0, 0.5, 0.25, 0.1, 0.01, 0.75], dtype=np.float32)
    lam = _check(w, 0.5, row_target=rt)[0].cpu().numpy()
    np.testing.assert_allclose(lam, 1.0 / rt, rtol=1e-5)


def test_full_size_sampled_rows_and_budget_is_met():
    T, target = 8192, 0.6
    _say(f"budget: bf16 T={T} V=151936 full size abar={target}: sampled rows + Z(lambda) = abar on every row")
    w = wl.rollout(DEV, T=T)
    lam, n = _check(w, target, rows=[0, 1, 63, 64, 4095, 4096, 8190, 8191])
    assert n == 8
    # Z_t(lambda_t) = sum_v min(q, p / lambda_t), recomputed with torch in float64, 256 rows at a time
    worst = 0.0
    for r0 in range(0, T, 256):
        q = torch.softmax(w.actor[r0:r0 + 256].double(), dim=1)
        p = torch.softmax(w.policy[r0:r0 + 256].double(), dim=1)
        z = torch.minimum(q, p / lam[r0:r0 + 256].double()[:, None]).sum(dim=1)
        worst = max(worst, float((z - target).abs().max()))
    assert worst < 1e-3 * target, worst


def test_bad_arguments():
    _say("budget: host-side validation")
    w = wl.tiny(DEV)
    buf = obrs.run_workload(w, 0)
    for bad in (0.0, -0.5, 1.01, float("nan")):
        with pytest.raises(obrs.JpError) as e:
            obrs.jp_obrs_lambda_for_budget(w.actor, w.policy, bad, buf)
        assert e.value.status == obrs.JP_ERR_PARAM
    small = obrs.Buffers(buf.out, buf.tensors, buf.workspace[:64])
    with pytest.raises(obrs.JpError) as e:
        obrs.jp_obrs_lambda_for_budget(w.actor, w.policy, 0.5, small)
    assert e.value.status == obrs.JP_ERR_WORKSPACE
    torch.cuda.synchronize()


# ---- one lambda for the whole batch: mean_t Z_t(lambda) = abar ---------------------------------------

def _zbar(w, lam, rows_per_step=256):
    """(1/n) sum_t Z_t(lambda) over the valid rows, float64 with torch, a slab of rows at a time."""
    tot, n = 0.0, 0
    for r0 in range(0, w.T, rows_per_step):
        sl = slice(r0, r0 + rows_per_step)
        ok = w.sampled_ids[sl] >= 0
        if not bool(ok.any()):
            continue
        q = torch.softmax(w.actor[sl][ok].double(), dim=1)
        p = torch.softmax(w.policy[sl][ok].double(), dim=1)
        tot += float(torch.minimum(q, p / lam).sum())
        n += int(ok.sum())
    return tot / n


def _check_batch(w, target, oracle=True):
    buf = obrs.run_workload(w, 0)
    lam = float(obrs.jp_obrs_lambda_for_budget_batch(w.actor, w.policy, target, buf).cpu()[0])
    tol = pu.TOL[w.actor.dtype]
    zmax = _zbar(w, 1e-30)
    assert abs(_zbar(w, lam) - min(target, zmax)) <= tol * target, (target, lam)
    if oracle:
        want = orc.lambda_for_budget_batch(wl.logits_to_numpy(w.actor), wl.logits_to_numpy(w.policy),
                                           w.sampled_ids.cpu().numpy(), target)
        # condition number of the problem from the slope of the mean: d lambda / lambda = -cond d abar / abar
        eps = 1e-4
        slope = (_zbar(w, want * (1 + eps)) - _zbar(w, want * (1 - eps))) / (2 * eps)     # dZ / dlog(lambda) < 0
        cond = target / max(-slope, 1e-300)
        if cond <= 100.0:
            assert abs(lam - want) <= tol * (1.0 + cond) * want, (target, lam, want, cond)
    return lam


@pytest.mark.parametrize("target", [1.0, 0.9, 0.5, 0.1, 1e-3])
def test_batch_tiny_config_fp32(target):
    _say(f"batch budget: tiny fp32 T=64 V=1024 abar={target}")
    _check_batch(wl.tiny(DEV), target)


def test_batch_rollout_shape_bf16_with_padding():
    _say("batch budget: bf16 T=24 V=151936, per-row noise, padding rows")
    w = wl.make_logits(24, wl.QWEN3_VOCAB, torch.bfloat16, seed=wl.BASE_SEED + 3, device=DEV,
                       noise_sigma_range=(0.1, 3.0), pad_every=6).with_params(k=8)
    prev = None
    for target in (0.8, 0.4, 0.05):
        lam = _check_batch(w, target)
        assert prev is None or lam > prev
        prev = lam


def test_batch_one_valid_row_equals_the_per_row_solver():
    _say("batch budget: a single valid row")
    w = wl.make_logits(5, 4100, torch.float32, seed=12, device=DEV, noise_sigma=1.0).with_params(k=8)
    w.sampled_ids[:] = -1
    w.sampled_ids[3] = 17
    buf = obrs.run_workload(w, 0)
    lam_b = float(obrs.jp_obrs_lambda_for_budget_batch(w.actor, w.policy, 0.3, buf).cpu()[0])
    lam_r = float(obrs.jp_obrs_lambda_for_budget(w.actor, w.policy, 0.3, buf).cpu()[3])
    assert lam_b == pytest.approx(lam_r, rel=1e-5)
    w.sampled_ids[:] = -1                                     # and none at all
    buf = obrs.run_workload(w, 0)
    assert np.isnan(float(obrs.jp_obrs_lambda_for_budget_batch(w.actor, w.policy, 0.3, buf).cpu()[0]))


def test_batch_full_size_budget_is_met():
    T, target = 8192, 0.6
    _say(f"batch budget: bf16 T={T} V=151936 full size abar={target}: mean Z(lambda) = abar")
    w = wl.rollout(DEV, T=T)
    lam = _check_batch(w, target, oracle=False)
    # repeatable to the bit: fixed-point sums do not depend on the order of the atomics
    buf = obrs.run_workload(w, 0)
    again = float(obrs.jp_obrs_lambda_for_budget_batch(w.actor, w.policy, target, buf).cpu()[0])
    assert again == lam
