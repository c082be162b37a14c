"""Rows split over two or four wavefronts (what the library does by itself for small batches of
long rows, in the two-tensor, stored-actor and vocabulary-chunked forms) against the oracle and
against the one-wave-per-row form of the same call (JP_FLAG_ONE_WAVE_PER_ROW): index lists and
union sizes must be identical, floats agree to the tolerance of the dtype."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl
    import parity_util as pu

DEV = "cuda"
FLAGS = 1 | 2                       # exact Z + top-k log-probabilities
KL = 8                              # + the distillation term (another instantiation of the kernel)
ONE = 32                            # JP_FLAG_ONE_WAVE_PER_ROW


def _say(msg):
    print(msg, flush=True)


def _same_as_one_wave(w, buf, flags=FLAGS):
    """The split form against the unsplit one: integers exactly, floats to the dtype's bar."""
    ref = obrs.run_workload(w, flags | ONE)
    torch.cuda.synchronize()
    tol = pu.TOL[w.actor.dtype]
    for name in ("topk_actor", "topk_policy", "union_size"):
        a, b = getattr(buf, name).cpu().numpy(), getattr(ref, name).cpu().numpy()
        assert np.array_equal(a, b), name
    # a token whose uniform sits within rounding of its acceptance probability may take either mask
    # value; the batch factor kappa, and with it every weight, then differs between the two runs
    same_mask = np.array_equal(buf.mask.cpu().numpy(), ref.mask.cpu().numpy())
    kl = ("distill_kl",) if flags & KL else ()
    for name in ("accept_prob", "z_approx", "z_exact") + kl + (("w_obrs", "rho") if same_mask else ()):
        a, b = getattr(buf, name).float().cpu().numpy(), getattr(ref, name).float().cpu().numpy()
        np.testing.assert_allclose(a, b, rtol=tol, atol=tol if name == "distill_kl" else 1e-30, equal_nan=True,
                                   err_msg=name)
    for name in ("logq", "logp", "logratio", "topk_actor_logq", "topk_policy_logp"):
        a, b = getattr(buf, name).float().cpu().numpy(), getattr(ref, name).float().cpu().numpy()
        fin = np.isfinite(a) & np.isfinite(b)
        assert np.array_equal(np.isfinite(a), np.isfinite(b)), name
        np.testing.assert_allclose(a[fin], b[fin], rtol=0, atol=tol, err_msg=name)
    return ref


def _case(seed):
    rng = np.random.default_rng(7000 + seed)
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    esz = 2 if dtype == torch.bfloat16 else 4
    vec = 16 // esz
    # two, four, eight ... sweep iterations of 64 chunks, around the boundaries of the waves' runs
    base = int(rng.choice([4 * 64 * vec, 8 * 64 * vec, 9 * 64 * vec, 16 * 64 * vec, 20000, 33333]))
    V = base + int(rng.integers(-3, 70))
    T = int(rng.integers(1, 24))
    k = int(rng.choice([1, 7, 63, 64, 65, 128, 129, 255, 256]))
    lam = float(rng.choice([0.3, 1.0, 1.7, 4.0]))
    stride = (V * esz + 15) // 16 * 16 // esz + vec * int(rng.integers(0, 3))
    quant = float(rng.choice([0.0, 0.0, 0.5, 2.0]))
    mask_frac = float(rng.choice([0.0, 0.0, 0.3]))
    return dict(seed=seed, dtype=dtype, V=V, T=T, k=k, lam=lam, stride=stride, quant=quant, mask_frac=mask_frac)


def _workload(c, seed):
    w = wl.make_logits(c["T"], c["V"], c["dtype"], seed=9000 + seed, device=DEV, actor_sigma=2.0,
                       spikes=3, noise_sigma=0.8, pad_every=6, row_stride=c["stride"])
    w = w.with_params(lam=c["lam"], k=c["k"])
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    V, T = c["V"], c["T"]
    if c["quant"] > 0:
        for t in (w.actor, w.policy):
            t[:, :V] = (torch.round(t[:, :V].float() / c["quant"]) * c["quant"]).to(c["dtype"])
    if c["mask_frac"] > 0:
        x = w.sampled_ids.clamp(min=0).long()
        for t, frac in ((w.actor, c["mask_frac"]), (w.policy, c["mask_frac"] / 2)):
            drop = torch.rand((T, V), generator=g, device=DEV) < frac
            drop[torch.arange(T, device=DEV), x] = False
            drop[:, 0] = False
            t[:, :V][drop] = float("-inf")
    w.ref_logprob = -torch.rand(T, generator=g, device=DEV) * 3.0
    return w


@pytest.mark.parametrize("seed", range(32))
def test_random_case_split(seed):
    c = _case(seed)
    _say({n: (str(v) if n == "dtype" else v) for n, v in c.items()})
    w = _workload(c, seed)
    flags = FLAGS | (KL if seed % 2 else 0)
    buf, R, st = pu.check_all(w, flags)
    _same_as_one_wave(w, buf, flags)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("k", [40, 128, 256])
def test_ties_across_the_runs_of_the_waves(dtype, k):
    """Constant rows, a few distinct values, monotone rows, the largest values all in one wave's run
    or in the ragged remainder: equal values must still rank by ascending id over the whole row."""
    _say(f"{dtype} k={k}: ties and placement across the waves' runs")
    T, V, pitch = 8, 20011, 20016                                         # ragged rows in 16-byte aligned storage
    a_store = torch.zeros((T, pitch), dtype=torch.float32, device=DEV)
    p_store = torch.zeros((T, pitch), dtype=torch.float32, device=DEV)
    a, p = a_store[:, :V], p_store[:, :V]
    g = torch.Generator(device=DEV); g.manual_seed(11)
    a[0] = 1.5; p[0] = -0.25                                              # constant rows
    a[1] = torch.randint(-2, 3, (V,), generator=g, device=DEV).float()    # five distinct values
    p[1] = torch.randint(-2, 3, (V,), generator=g, device=DEV).float()
    a[2] = -torch.arange(V, device=DEV).float() * 0.002                   # all of the best in the first run
    p[2] = torch.arange(V, device=DEV).float() * 0.002                    # all of the best in the last run / remainder
    a[3] = torch.randn(V, generator=g, device=DEV)
    a[3, V - 300:] += 9.0                                                 # the best in the ragged end
    p[3] = torch.randn(V, generator=g, device=DEV)
    p[3, V // 2 - 150: V // 2 + 150] += 9.0                               # the best straddle a boundary of two runs
    a[4, :] = float("-inf"); a[4, 15000:15030] = 0.0                      # fewer finite entries than k
    p[4] = torch.randn(V, generator=g, device=DEV)
    a[5] = torch.randn(V, generator=g, device=DEV); p[5] = a[5]           # matched distributions
    a[6] = 0.0; a[6, ::977] = 1.0                                         # a plateau above a plateau
    p[6] = 0.0; p[6, 5::1201] = 1.0
    a[7] = torch.randn(V, generator=g, device=DEV) * 30.0                 # the exponent reference moves often
    p[7] = torch.randn(V, generator=g, device=DEV) * 30.0
    x = torch.tensor([17, 3, 19000, 19990, 15010, 4010, 977, 5], dtype=torch.int32, device=DEV)
    u = torch.tensor([0.3, 0.6, 0.999, 0.01, 0.5, 0.2, 0.7, 0.4], dtype=torch.float32, device=DEV)
    w = wl.Workload("degenerate", a_store.to(dtype)[:, :V], p_store.to(dtype)[:, :V], x, u, lam=2.0, k=k)
    buf, R, st = pu.check_all(w, FLAGS)
    assert buf.topk_actor[0].cpu().tolist() == list(range(k))
    assert buf.topk_actor[2].cpu().tolist() == list(range(k))
    if dtype == torch.float32:                                            # (bf16 rounds neighbours to equal values)
        assert buf.topk_policy[2].cpu().tolist() == list(range(V - 1, V - 1 - k, -1))
    _same_as_one_wave(w, buf)


@pytest.mark.parametrize("T", [1792, 1793])
def test_batch_sizes_around_the_switch(T):
    """Rows are split up to T = 1792 and not beyond: the oracle on every row."""
    V, k = 4099, 20
    _say(f"bf16 T={T} V={V} k={k}")
    w = wl.make_logits(T, V, torch.bfloat16, seed=31 + T, device=DEV, actor_sigma=2.0, spikes=3,
                       noise_sigma=0.8, pad_every=97, row_stride=4104).with_params(lam=1.3, k=k)
    buf, R, st = pu.check_all(w, FLAGS)
    _same_as_one_wave(w, buf)


@pytest.mark.parametrize("dtype,T", [(torch.bfloat16, 1024), (torch.bfloat16, 1700), (torch.float32, 512)])
def test_vocabulary_of_the_named_workloads(dtype, T):
    """V = 151936 at batch sizes that are split: sampled rows against the oracle, every row against
    the one-wave form."""
    _say(f"{dtype} T={T} V=151936 k=64")
    w = wl.make_logits(T, wl.QWEN3_VOCAB, dtype, seed=wl.BASE_SEED + 40 + T, device=DEV,
                       noise_sigma=1.0).with_params(k=64)
    buf = obrs.run_workload(w, FLAGS)
    torch.cuda.synchronize()
    _same_as_one_wave(w, buf)
    rows = np.unique(np.linspace(0, T - 1, 24).astype(np.int64))
    R = pu.run_oracle(w, rows=rows)
    pu.check_rows(buf, w, R, rows=rows, flags=FLAGS)


@pytest.mark.parametrize("seed", range(12))
def test_random_case_split_stored_actor_side(seed):
    """The stored-actor form splits its rows by the same rule: against the oracle in both forms, and
    the two forms against each other."""
    import test_gpu_stored as stored_form
    c = _case(100 + seed)
    rule = seed % 3
    _say({n: (str(v) if n == "dtype" else v) for n, v in c.items()} | {"rule": rule})
    w = _workload(c, 100 + seed)
    stored = stored_form.stored_side(w, w.k)
    buf, R, st = stored_form.run_case(w, rule, 2, *stored)
    ref, R1, st1 = stored_form.run_case(w, rule, 2 | ONE, *stored)
    tol = pu.TOL[w.actor.dtype]
    for name in ("topk_policy", "union_size"):
        assert np.array_equal(getattr(buf, name).cpu().numpy(), getattr(ref, name).cpu().numpy()), name
    for name in ("accept_prob", "z_approx"):
        np.testing.assert_allclose(getattr(buf, name).cpu().numpy(), getattr(ref, name).cpu().numpy(), rtol=tol,
                                   atol=1e-30, equal_nan=True, err_msg=name)


@pytest.mark.parametrize("T,V,da,dp,k,chunk", [
    (40, 9000, 128, 192, 20, 1024),      # groups of 4096 columns: four waves, then a ragged last group
    (21, 9000, 64, 128, 200, 512),       # k class 256: two waves
    (130, 5000, 64, 64, 64, 256),        # groups of 1024 columns: two waves
    (9, 30000, 64, 64, 128, 0),          # one wide chunk, four waves, no carried record at all
])
def test_chunked_forms_split_rows_too(T, V, da, dp, k, chunk):
    """The vocabulary-chunked forms (logits from the matrix cores, row records carried between
    launches) split their rows by the same rule: against the oracle, and against the one-wave form of
    the same call, whose GEMM output is bit-identical, so the index lists must be too."""
    import test_gpu_lmhead as lm
    import test_gpu_lmhead_stored as lms
    _say(f"lm_head T={T} V={V} d=({da},{dp}) k={k} chunk={chunk}")
    w = wl.lm_head(T, V, da, dp, DEV, seed=300 + T, k=k).with_params(lam=0.8)
    w.ref_logprob = -torch.rand(T, device=DEV)
    flags = obrs.JP_FLAG_TOPK_LOGPROBS | obrs.JP_FLAG_DISTILL_KL
    buf = lm._run(w, flags, chunk)
    lm._check(w, buf, np.arange(T), flags)
    ref = lm._run(w, flags | ONE, chunk)
    for name in ("topk_actor", "topk_policy", "union_size"):
        assert torch.equal(buf.tensors[name], ref.tensors[name]), name
    for name in ("accept_prob", "z_approx", "logq", "logp", "distill_kl", "topk_actor_logq", "topk_policy_logp"):
        np.testing.assert_allclose(buf.tensors[name].cpu().numpy(), ref.tensors[name].cpu().numpy(),
                                   rtol=1e-5, atol=1e-5, err_msg=name)
    rows = np.arange(T)
    got, _ = lms.run_case(w, 1, rows, flags=obrs.JP_FLAG_TOPK_LOGPROBS, vocab_chunk=chunk)
    one, _ = lms.run_case(w, 1, rows, flags=obrs.JP_FLAG_TOPK_LOGPROBS | ONE, vocab_chunk=chunk)
    for name in ("topk_policy", "union_size"):
        assert torch.equal(got.tensors[name], one.tensors[name]), name
    for name in ("accept_prob", "z_approx", "logp"):
        np.testing.assert_allclose(got.tensors[name].cpu().numpy(), one.tensors[name].cpu().numpy(),
                                   rtol=1e-5, atol=1e-5, err_msg=name)
