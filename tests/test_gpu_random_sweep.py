"""Seeded random sweep of small shapes through the C ABI against the oracle: vocabulary sizes around
the chunk, iteration and tile boundaries, every k class, both dtypes, padded strides, padding rows,
heavy ties (logits quantised to a few values) and masked (-inf) entries."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl
    import parity_util as pu
    import test_gpu_stored as stored_form
    import test_gpu_budget as budget

DEV = "cuda"
ALL_FLAGS = 1 | 2 | 8


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    esz = 2 if dtype == torch.bfloat16 else 4
    vec = 16 // esz
    base = int(rng.choice([1, vec, 64 * vec, 128 * vec, 1000, 4096, 20000]))
    V = max(1, base + int(rng.integers(-3, 4)))
    T = int(rng.integers(1, 40))
    k = int(min(V, rng.choice([1, 2, 7, 63, 64, 65, 128, 129, 255, 256])))
    lam = float(rng.choice([0.3, 1.0, 1.7, 4.0]))
    stride = (V * esz + 15) // 16 * 16 // esz + (16 // esz) * int(rng.integers(0, 3))
    quant = float(rng.choice([0.0, 0.0, 0.5, 2.0]))          # > 0: logits rounded to multiples of it (ties)
    mask_frac = float(rng.choice([0.0, 0.0, 0.3]))
    return dict(seed=seed, dtype=dtype, V=V, T=T, k=k, lam=lam, stride=stride, quant=quant, mask_frac=mask_frac)


def _workload(c, seed):
    w = wl.make_logits(c["T"], c["V"], c["dtype"], seed=5000 + seed, device=DEV, actor_sigma=2.0,
                       spikes=min(3, c["V"]), noise_sigma=0.8, pad_every=6, row_stride=c["stride"])
    w = w.with_params(lam=c["lam"], k=c["k"])
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    if c["quant"] > 0:
        for t in (w.actor, w.policy):
            t[:, : c["V"]] = (torch.round(t[:, : c["V"]].float() / c["quant"]) * c["quant"]).to(c["dtype"])
    if c["mask_frac"] > 0 and c["V"] > 4:
        drop = torch.rand((c["T"], c["V"]), generator=g, device=DEV) < c["mask_frac"]
        x = w.sampled_ids.clamp(min=0).long()
        drop[torch.arange(c["T"], device=DEV), x] = False     # the sampled token stays possible
        drop[:, 0] = False
        w.actor[:, : c["V"]][drop] = float("-inf")
        drop2 = torch.rand((c["T"], c["V"]), generator=g, device=DEV) < c["mask_frac"] / 2
        drop2[torch.arange(c["T"], device=DEV), x] = False
        drop2[:, 0] = False
        w.policy[:, : c["V"]][drop2] = float("-inf")
    w.ref_logprob = -torch.rand(c["T"], generator=g, device=DEV) * 3.0
    return w


@pytest.mark.parametrize("seed", range(40))
def test_random_case(seed):
    c = _case(seed)
    print({n: (str(v) if n == "dtype" else v) for n, v in c.items()}, flush=True)
    pu.check_all(_workload(c, seed), ALL_FLAGS)


@pytest.mark.parametrize("seed", range(40, 64))
def test_random_case_stored_actor_side(seed):
    """The same kind of case through jp_obrs_forward_stored, the stored side taken from the actor row
    (its top-k by (value desc, id asc), in float64 on the host), one of the three tail rules."""
    c = _case(seed)
    rule = seed % 3
    print({n: (str(v) if n == "dtype" else v) for n, v in c.items()}, "rule", rule, flush=True)
    stored_form.run_case(_workload(c, seed), rule, flags=2)


# 287 .. 660: fp32 logits rounded to multiples of 2, so a row has a handful of distinct ratios and
# thousands of equal terms meet in one histogram bin (sums in fp32 drift there: the bins are float64)
@pytest.mark.parametrize("seed", list(range(64, 88)) + [287, 380, 532, 589, 660])
def test_random_case_budget(seed):
    """The same kind of case through jp_obrs_lambda_for_budget with a random budget per row, and
    through the per-batch solver with one random budget."""
    c = _case(seed)
    print({n: (str(v) if n == "dtype" else v) for n, v in c.items()}, flush=True)
    w = _workload(c, seed)
    rng = np.random.default_rng(seed)
    targets = rng.choice([1.0, 0.999, 0.9, 0.5, 0.2, 0.01], size=c["T"]).astype(np.float32)
    budget._check(w, 0.5, row_target=targets)
    if bool((w.sampled_ids >= 0).any()):
        budget._check_batch(w, float(rng.choice([0.9, 0.5, 0.1])))
