"""GPU parity of jp_obrs_distill_grad (gradient of the distillation term w.r.t. the actor logits,
Sec. 4.2 (3)) against the float64 oracle, element by element.

Tolerance: the gradient is a difference of two probabilities, so the bound is taken relative to
the larger of them: |g - g*| <= tol |w| max(q, p) with tol = 1e-5 for fp32 logits and 1e-3 for
bf16 logits.  A bf16 gradient is additionally allowed the rounding of its own storage format
(half a unit in the last place, 2^-9 relative)."""
import numpy as np
import pytest
import scipy.special
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from oracle import obrs_oracle as orc
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl

DEV = "cuda"
TOL = {torch.float32: 1e-5, torch.bfloat16: 1e-3}


def _say(msg):
    print(msg, flush=True)


def _grad_to_f64(g: torch.Tensor) -> np.ndarray:
    return g.float().cpu().numpy().astype(np.float64)


def _check(w, grad_dtype, row_scale=None, scale=1.0, rows=None, grad_stride=None):
    """Forward (leaves the log-sum-exps in the workspace), gradient, comparison on `rows`."""
    T, V = w.T, w.V
    buf = obrs.run_workload(w, 0)
    gs = V if grad_stride is None else grad_stride
    store = torch.full((T, gs), float("nan"), dtype=grad_dtype, device=DEV)
    grad = store[:, :V]
    rs = None if row_scale is None else torch.as_tensor(row_scale, dtype=torch.float32, device=DEV)
    obrs.jp_obrs_distill_grad(w.actor, w.policy, rs, scale, grad, buf)
    torch.cuda.synchronize()
    if gs > V:
        assert torch.isnan(store[:, V:].float()).all(), "wrote past the end of a row"
    idx = np.arange(T) if rows is None else np.asarray(rows)
    sel = torch.as_tensor(idx, device=DEV)
    a = wl.logits_to_numpy(w.actor[sel])
    p = wl.logits_to_numpy(w.policy[sel])
    x = w.sampled_ids[sel].cpu().numpy()
    rs_np = None if row_scale is None else np.asarray(row_scale, dtype=np.float32)[idx]
    want = orc.distill_grad(a, p, x, rs_np, scale)
    got = _grad_to_f64(grad[sel])
    a64 = wl.logits_to_float64(w.actor[sel])
    p64 = wl.logits_to_float64(w.policy[sel])
    tol = TOL[w.actor.dtype]
    for i in range(len(idx)):
        if x[i] < 0 or x[i] >= V:
            assert np.all(got[i] == 0.0), f"row {idx[i]} takes no part in the loss"
            continue
        wt = abs(scale * (1.0 if rs_np is None else float(rs_np[i])))
        big = np.maximum(scipy.special.softmax(a64[i]), scipy.special.softmax(p64[i]))
        bound = tol * wt * big + 1e-30
        if grad_dtype == torch.bfloat16:
            bound = bound + np.abs(want[i]) * 2.0 ** -8 + 1e-38
        err = np.abs(got[i] - want[i])
        j = int(np.argmax(err - bound))
        assert err[j] <= bound[j], (f"row {idx[i]} id {j}: got {got[i, j]!r} want {want[i, j]!r} "
                                    f"bound {bound[j]!r}")
    return grad, buf


@pytest.mark.parametrize("grad_dtype", [torch.float32, torch.bfloat16])
def test_tiny_config_fp32(grad_dtype):
    _say(f"distill grad: tiny fp32 T=64 V=1024 -> {grad_dtype}")
    _check(wl.tiny(DEV), grad_dtype, scale=1.0 / 64)


@pytest.mark.parametrize("grad_dtype", [torch.float32, torch.bfloat16])
def test_rollout_shape_bf16(grad_dtype):
    _say(f"distill grad: bf16 T=24 V=151936 -> {grad_dtype}, per-row weights")
    w = wl.make_logits(24, wl.QWEN3_VOCAB, torch.bfloat16, seed=wl.BASE_SEED + 1, device=DEV,
                       noise_sigma=1.0).with_params(k=64)
    rs = np.linspace(-1.0, 2.0, 24).astype(np.float32)
    _check(w, grad_dtype, row_scale=rs, scale=0.5)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 37, 255, 515, 1027, 4100, 33333])
def test_ragged_shapes_padding_and_strides(dtype, V):
    T = 13
    _say(f"distill grad: {dtype} T={T} V={V}, padded strides, padding rows, a bad id")
    esz = 2 if dtype == torch.bfloat16 else 4
    stride = (V * esz + 15) // 16 * 16 // esz + 16 // esz * 3
    w = wl.make_logits(T, V, dtype, seed=4321 + V, device=DEV, actor_sigma=2.0, spikes=min(3, V),
                       noise_sigma=0.7, pad_every=5, row_stride=stride).with_params(k=min(V, 8))
    w.sampled_ids[7] = V + 5                          # outside the vocabulary: row dropped from the loss
    for gd in (torch.float32, torch.bfloat16):
        gsz = 2 if gd == torch.bfloat16 else 4
        gstride = (V * gsz + 15) // 16 * 16 // gsz + 16 // gsz
        _check(w, gd, row_scale=np.full(T, 1.5, np.float32), scale=-2.0, grad_stride=gstride)


def test_matched_distributions_give_zero():
    _say("distill grad: p == q -> exactly zero")
    w = wl.make_logits(5, 3000, torch.bfloat16, seed=3, device=DEV)
    w = w.with_params(policy=w.actor.clone(), k=8)
    grad, _ = _check(w, torch.float32)
    assert torch.all(grad == 0)


def test_full_size_sampled_rows_and_zero_sum():
    T = 8192
    _say(f"distill grad: bf16 T={T} V=151936 full size, sampled rows + per-row zero sum")
    w = wl.rollout(DEV, T=T)
    rows = [0, 1, 63, 64, 4095, 4096, 8190, 8191]
    grad, _ = _check(w, torch.bfloat16, scale=1.0 / T, rows=rows)
    del grad
    store = torch.empty((T, w.V), dtype=torch.float32, device=DEV)
    buf = obrs.run_workload(w, 0)
    obrs.jp_obrs_distill_grad(w.actor, w.policy, None, 1.0, store, buf)
    torch.cuda.synchronize()
    # sum_v (q - p) = 0: every row, at any size; the sum of 151936 fp32 terms of size <= 1 leaves ~1e-5
    s = store.double().sum(dim=1).abs().max().item()
    assert s < 1e-4, s
    a = store.abs().sum(dim=1)
    assert torch.all(a > 0) and torch.all(a <= 2.0 + 1e-3)      # ||q - p||_1 <= 2


def test_training_size_sampled_rows_and_zero_sum():
    T = 65536
    _say(f"distill grad: bf16 T={T} V=151936 (the training batch: 4.9 M workgroups), sampled rows + zero sum")
    w = wl.training(DEV)
    rows = [0, 1, 4095, 4096, 32767, 32768, 65534, 65535]
    grad, _ = _check(w, torch.bfloat16, scale=1.0, rows=rows)
    # sum_v (q - p) = 0 on every row; bf16 storage rounds each entry by <= 2^-9 of itself and
    # sum_v |q - p| <= 2, so the row sum stays below 2 * 2^-9
    worst = 0.0
    for a in range(0, T, 4096):
        worst = max(worst, grad[a:a + 4096].double().sum(dim=1).abs().max().item())
    assert worst < 2.0 * 2.0 ** -9, worst
    del grad, w
    torch.cuda.empty_cache()


def test_bad_arguments():
    _say("distill grad: host-side validation")
    w = wl.tiny(DEV)
    buf = obrs.run_workload(w, 0)
    T, V = w.T, w.V
    g = torch.empty((T, V), dtype=torch.float32, device=DEV)
    lib = obrs.raw()
    import ctypes as C

    def call(actor=w.actor.data_ptr(), grad=g.data_ptr(), gstride=V, gdt=obrs.JP_F32, scale=1.0,
             ws=buf.workspace.data_ptr(), wsb=buf.workspace.numel(), stride=V):
        return lib.jp_obrs_distill_grad(C.c_void_p(actor), C.c_void_p(w.policy.data_ptr()), T, V, stride,
                                        obrs.JP_F32, None, C.c_float(scale), C.c_void_p(grad), gstride, gdt,
                                        C.c_void_p(ws), wsb, None)

    assert call() == obrs.JP_OK
    assert call(grad=None) == obrs.JP_ERR_NULL
    assert call(grad=g.data_ptr() + 4) == obrs.JP_ERR_ALIGN
    assert call(gstride=V - 1) == obrs.JP_ERR_SHAPE
    assert call(gstride=V + 1) == obrs.JP_ERR_ALIGN
    assert call(gdt=9) == obrs.JP_ERR_UNSUPPORTED
    assert call(scale=float("nan")) == obrs.JP_ERR_PARAM
    assert call(wsb=64) == obrs.JP_ERR_WORKSPACE
    assert call(stride=V - 8) == obrs.JP_ERR_SHAPE
    torch.cuda.synchronize()
