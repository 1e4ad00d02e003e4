"""GPU parity of mts_attn_pointwise against the oracle's attn_pointwise, through every kernel
that serves it: the plain fp32 kernel, the streaming matrix-core kernel under several work
schedules (cut pairs are finished by adding pieces) and the workgroup-per-query-block kernel.
Tolerances as for the softmax form: fp32 max-abs 1e-5 (relative to max |oracle| where that
exceeds 1), bf16 2e-2 of max |oracle| per (user, head)."""
import numpy as np
import pytest

import mts_workloads as W
import oracle
from helpers import draw_step_data, as_values
from test_gpu_parity import CASES, PREFILL_CASES, SCHEDULES, FILL, _case, _oracle_store

from conftest import KERNEL_PLAIN, KERNEL_PREFILL, KERNEL_STREAMING  # noqa: F401

pytestmark = pytest.mark.gpu


def _check(w, got, ref):
    gv = as_values(got)
    assert np.isfinite(gv).all(), "non-finite output"
    worst = 0.0
    for u in range(w.batch):
        lo, hi = int(w.new_indptr[u]), int(w.new_indptr[u + 1])
        if hi == lo:
            continue
        for h in range(w.heads):
            r = ref[lo:hi, h]
            scale = max(1.0, np.abs(r).max())
            tol = 1e-5 * scale if w.dtype == "f32" else 2e-2 * np.abs(r).max()
            err = np.abs(gv[lo:hi, h] - r).max()
            assert err <= tol, f"user {u} head {h}: err {err:.3e} > tol {tol:.3e}"
            worst = max(worst, err / tol)
    return worst


def _run(w, inv_norm, sm_scale=0.0):
    import gpu_harness as G
    data = draw_step_data(w)
    step = G.GpuStep(w, fill_byte=FILL)
    store = _oracle_store(w, data)
    for l in range(w.layers):
        step.unpack_histories(data, l)
        step.append(data, l)
        got = step.attention_pointwise(data, l, inv_norm, sm_scale)
        ref = oracle.attn_pointwise(store, l, data["q"][l], w.page_indptr, w.page_indices, w.prefix_lens,
                                    w.new_indptr, inv_norm, sm_scale=(sm_scale or None))
        _check(w, got, ref)


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("schedule", list(SCHEDULES))
def test_pointwise_small(name, schedule, attn_tuning):
    attn_tuning(**SCHEDULES[schedule])
    w = _case(name)
    _run(w, inv_norm=1.0 / max(1, int(w.total_lens.max())))


@pytest.mark.parametrize("name", list(PREFILL_CASES))
def test_pointwise_long_new_segments(name):
    dtype, L, H, D, S, prefix, new, chunk = PREFILL_CASES[name]
    w = W.custom_workload(name, 200 + len(name), dtype, L, H, D, S, prefix, new, chunk_tokens=chunk)
    _run(w, inv_norm=1.0 / int(w.total_lens.max()), sm_scale=0.11)


@pytest.mark.parametrize("name", ["bf16_ragged", "bf16_d128_s32", "bf16_empty_users"])
def test_pointwise_small_through_the_prefill_kernel(name, attn_tuning):
    attn_tuning(kernel=KERNEL_PREFILL)
    _run(_case(name), inv_norm=0.02)


def test_pointwise_plain_kernel_agrees(attn_tuning):
    attn_tuning(kernel=KERNEL_PLAIN)
    _run(_case("bf16_ragged"), inv_norm=0.05, sm_scale=0.2)


def test_pointwise_is_not_softmax():
    """With zero queries the pointwise form gives exactly 0, the softmax form the mean of V."""
    import torch
    import gpu_harness as G
    w = _case("bf16_ragged")
    data = draw_step_data(w, layers=[0])
    data["q"][0] = np.zeros_like(data["q"][0])
    step = G.GpuStep(w, fill_byte=FILL)
    step.unpack_histories(data, 0)
    step.append(data, 0)
    assert np.all(as_values(step.attention_pointwise(data, 0, 1.0)) == 0.0)
    assert np.abs(as_values(step.attention(data, 0))).max() > 0.0
