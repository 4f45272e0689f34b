"""GPU parity of the token-granular recovery ratio (Section 2.4: the sum of a query's k largest
attention weights) against the oracle, through the C ABI."""
import time

import numpy as np
import pytest
import torch

import paper_2603_10353_amd as S
from oracle import shplb_oracle as orc
from workloads import bf16_bits_from_f32, make_custom, make_workload

from checks import TOKEN_RECOVERY_ATOL, TOKEN_RECOVERY_RTOL

pytestmark = pytest.mark.gpu


def _run(wl, budgets, softmax_scale=0.0):
    from harness import DevicePass
    print("case", wl.name, "seqlens", np.diff(wl.cu_seqlens).tolist(), "heads", wl.n_q_heads, wl.n_kv_heads,
          "block", wl.block, "budgets", list(budgets), flush=True)
    run = DevicePass(wl, softmax_scale=softmax_scale)
    run.token_recovery_step(budgets)
    torch.cuda.synchronize()
    return run, run.token_recovery.cpu().numpy()


@pytest.mark.parametrize("block", [64, 128])
@pytest.mark.parametrize("budgets", [[16], [1, 40], [3, 64, 65, 200], [1, 2, 8, 33, 128, 129, 500, 100000]])
def test_every_query_of_a_ragged_varlen_batch(block, budgets):
    wl = make_custom([5 * block + 37, 1, block - 3, 2 * block, 3 * block + 1], 8, 2, block,
                     [2] * 8, seed=71, name="token_recovery_b%d" % block)
    run, got = _run(wl, budgets)
    want = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets)
    assert not np.isnan(got).any()
    np.testing.assert_allclose(got, want, rtol=TOKEN_RECOVERY_RTOL, atol=TOKEN_RECOVERY_ATOL)
    heads = S.shplb_token_recovery_heads(run.p, got)
    np.testing.assert_allclose(heads, orc.token_recovery_heads(want), rtol=TOKEN_RECOVERY_RTOL)
    assert (np.diff(heads, axis=1) >= -1e-7).all()                 # more keys never hold less


def test_equal_weights_are_ties_at_the_threshold():
    # all keys equal: every weight of a query ties with its k-th largest; the k best hold min(k, t+1)/(t+1)
    T, block = 700, 128
    rng = np.random.default_rng(4)
    wl = make_custom([T], 2, 1, block, [2, 2], seed=1, name="token_recovery_ties")
    wl.k = bf16_bits_from_f32(np.tile(rng.standard_normal((1, 1, 128)).astype(np.float32), (T, 1, 1)))
    budgets = [1, 100, 699]
    _, got = _run(wl, budgets)
    t = np.arange(T)
    for b, kk in enumerate(budgets):
        want = np.minimum(kk, t + 1) / (t + 1.0)
        np.testing.assert_allclose(got[b], np.tile(want, (2, 1)), rtol=TOKEN_RECOVERY_RTOL)


def test_one_dominant_key_and_a_custom_scale():
    # a sharp softmax (large scale): the best key alone holds nearly everything, log-weights span hundreds
    wl = make_custom([900], 4, 4, 128, [2] * 4, seed=9, name="token_recovery_sharp")
    budgets = [1, 2, 50]
    _, got = _run(wl, budgets, softmax_scale=1.5)
    want = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets, softmax_scale=1.5)
    np.testing.assert_allclose(got, want, rtol=TOKEN_RECOVERY_RTOL, atol=TOKEN_RECOVERY_ATOL)
    assert np.median(got[0]) > 0.9


def test_is_deterministic():
    wl = make_workload(1, seqlens=[3000])
    run, a = _run(wl, [256])
    run.token_recovery_step([256])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a, run.token_recovery.cpu().numpy())


def test_32k_layer_at_the_profiled_budget_on_sampled_queries():
    # The setting of Section 2.4: a 32K context, k = 4096 tokens, one figure per head.  Sampled queries
    # against the oracle (first and last query, both sides of the budget, random ones); every value in (0, 1].
    wl = make_workload(1)
    T = int(wl.cu_seqlens[-1])
    budgets = [4096]
    run, got = _run(wl, budgets)
    t0 = time.perf_counter()
    run.token_recovery_step(budgets)
    torch.cuda.synchronize()
    print("  32K, k = 4096: %.1f ms" % ((time.perf_counter() - t0) * 1e3), flush=True)
    assert not np.isnan(got).any() and (got > 0).all() and (got <= 1 + 1e-5).all()
    np.testing.assert_array_equal(got[0][:, :4096], 1.0)           # these queries see at most 4096 keys
    rng = np.random.default_rng(12)
    tokens = sorted({0, 4095, 4096, 4097, T - 1} | set(rng.integers(4096, T, size=40).tolist()))
    want = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets, tokens=tokens)
    np.testing.assert_allclose(got[:, :, tokens], want[:, :, tokens], rtol=TOKEN_RECOVERY_RTOL, atol=TOKEN_RECOVERY_ATOL)
    heads = S.shplb_token_recovery_heads(run.p, got)
    print("  recovery per head at k = 4096:", np.round(heads[:, 0], 3), flush=True)
    assert heads.min() > 0.125 and heads.max() <= 1 + 1e-5        # a head recovers at least k/T by taking any k keys


def test_128k_layer_two_budgets_on_sampled_queries():
    # the longest context of the evaluation: 1024 key blocks per row, two budgets in one call
    wl = make_workload(2)
    T = int(wl.cu_seqlens[-1])
    budgets = [1024, 4096]
    run, got = _run(wl, budgets)
    assert not np.isnan(got).any() and (got > 0).all() and (got <= 1 + 1e-5).all()
    np.testing.assert_array_equal(got[0][:, :1024], 1.0)
    np.testing.assert_array_equal(got[1][:, :4096], 1.0)
    worst = float((got[0] - got[1]).max())
    print("  largest amount by which 1024 keys exceed 4096 keys: %.3g" % worst, flush=True)
    assert worst <= 2e-5                                           # more keys never hold less (fp32 sums of 4096 terms)
    rng = np.random.default_rng(13)
    tokens = sorted({1023, 1024, 4096, T - 1} | set(rng.integers(4096, T, size=20).tolist()))
    want = orc.token_recovery(wl.q, wl.k, wl.cu_seqlens, budgets, tokens=tokens)
    np.testing.assert_allclose(got[:, :, tokens], want[:, :, tokens], rtol=TOKEN_RECOVERY_RTOL, atol=TOKEN_RECOVERY_ATOL)
