"""jp_obrs_forward_static (the entry point that allocates nothing: its scratch is a static device
array inside the library) against jp_obrs_forward with a caller's workspace, through the C ABI.
Same kernels, so every output must agree bit for bit.  Two calls in a row share the one array; the
second is smaller, so whatever the first left behind must not leak into it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl
    import parity_util as pu

DEV = "cuda"
FLAGS = 1 | 2 | 8            # exact Z, top-k log-probabilities, distillation KL
# outputs the caller does not ask for live in the scratch instead
WANT_FEW = ["w_obrs", "rho", "mask", "union_size", "topk_actor", "topk_policy", "stats", "z_exact", "distill_kl"]


def _same(a, b, what):
    for n in a.tensors:
        x, y = a.tensors[n], b.tensors[n]
        ok = torch.equal(x, y) or (x.is_floating_point() and torch.equal(torch.nan_to_num(x), torch.nan_to_num(y)))
        assert ok, (what, n)


def _pair(w, flags, want=None):
    T, V, dt = w.T, w.V, obrs._dtype_code(w.actor)
    ref = obrs.alloc_buffers(T, V, w.k, dt, flags, DEV, want)
    obrs.jp_obrs_forward(w.actor, w.policy, w.sampled_ids, w.uniforms, w.ref_logprob, w.lam, w.k, w.c1, w.c2,
                         flags, ref)
    got = obrs.alloc_buffers(T, V, w.k, dt, flags, DEV, want)
    for t in got.tensors.values():
        t.fill_(0x5a if t.dtype == torch.uint8 else 7)
    got.workspace.fill_(0xee)                   # never passed to the call; must stay as it is
    obrs.jp_obrs_forward_static(w.actor, w.policy, w.sampled_ids, w.uniforms, w.ref_logprob, w.lam, w.k, w.c1,
                                w.c2, flags, got)
    torch.cuda.synchronize()
    assert bool((got.workspace == 0xee).all())
    return ref, got


def test_two_calls_in_a_row_the_second_smaller():
    print("static scratch: bf16 T=600 V=20011 k=64, then fp32 T=37 V=1027 k=24 with padding rows", flush=True)
    big = wl.make_logits(600, 20011, torch.bfloat16, seed=31, device=DEV, row_stride=20016).with_params(k=64, lam=0.8)
    big.ref_logprob = -torch.rand(big.T, device=DEV)
    ref, got = _pair(big, FLAGS, WANT_FEW)
    _same(ref, got, "first call")
    st = got.stats()
    assert st.n_valid == big.T and st.error_flags == 0

    small = wl.make_logits(37, 1027, torch.float32, seed=32, device=DEV, actor_sigma=2.0, spikes=3,
                           pad_every=5, row_stride=1032).with_params(k=24, lam=1.3)
    ref2, got2 = _pair(small, FLAGS)
    _same(ref2, got2, "second, smaller call")
    assert got2.stats().n_valid == ref2.stats().n_valid == 37 - 7
    # and against the oracle, to the usual bars
    R = pu.run_oracle(small)
    g, _ = pu.check_rows(got2, small, R, flags=FLAGS)
    pu.check_batch(got2, small, R, g, flags=FLAGS)

    # the first size again: the scratch now holds the small call's leftovers
    ref3, got3 = _pair(big, 0, WANT_FEW)
    _same(ref3, got3, "third call")


def test_empty_batch_and_size_limit():
    w = wl.make_logits(4, 128, torch.float32, seed=12, device=DEV, spikes=0).with_params(k=4)
    w0 = wl.Workload("empty", w.actor[:0], w.policy[:0], w.sampled_ids[:0], w.uniforms[:0], k=4)
    buf = obrs.alloc_buffers(0, 128, 4, obrs.JP_F32, 0, DEV)
    obrs.jp_obrs_forward_static(w0.actor, w0.policy, w0.sampled_ids, w0.uniforms, None, 1.0, 4, 3.0, 3.0, 0, buf)
    torch.cuda.synchronize()
    assert buf.stats().error_flags == obrs.JP_DATA_ERR_EMPTY
    # one row more than the scratch holds: refused with its own status, nothing launched
    T = obrs.JP_STATIC_MAX_T + 1
    a = torch.zeros((T, 8), dtype=torch.float32, device=DEV)
    ids = torch.zeros(T, dtype=torch.int32, device=DEV)
    big = obrs.alloc_buffers(T, 8, 2, obrs.JP_F32, 0, DEV, want=["w_obrs", "stats"])
    big.w_obrs.fill_(5.0)
    with pytest.raises(obrs.JpError) as e:
        obrs.jp_obrs_forward_static(a, a, ids, None, None, 1.0, 2, 3.0, 3.0, 0, big)
    assert e.value.status == obrs.JP_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert bool((big.w_obrs == 5.0).all())
    # exactly the maximum is served
    ok = obrs.alloc_buffers(T - 1, 8, 2, obrs.JP_F32, 0, DEV, want=["w_obrs", "stats"])
    obrs.jp_obrs_forward_static(a[:T - 1], a[:T - 1], ids[:T - 1], None, None, 1.0, 2, 3.0, 3.0, 0, ok)
    torch.cuda.synchronize()
    st = ok.stats()
    assert st.n_valid == T - 1 and st.error_flags == 0
    assert abs(st.mean_z_approx - 2.0 / 8.0) < 1e-6     # constant rows: Z_approx = k / V
