"""Comparison rules shared by the GPU parity tests (tolerances stated here)."""
from __future__ import annotations

import numpy as np

SCORE_ATOL = 2e-5      # fp32 pooling + fp32 dot of 128 terms against the fp64 oracle
SEL_WAIVER = 1e-5      # a swap is allowed only between scores this close to the row's threshold
OUT_MAX_ABS = 2e-2     # bf16 inputs, bf16 P, fp32 accumulate
OUT_MAX_REL = 1e-2     # max|diff| / max|oracle| per head
MASS_RTOL = 2e-4      # block mass: fp32 exp2 of fp32 logits (|s| of a few tens) and fp32 sums of up to 16K terms
MASS_ATOL = 1e-7
TOKEN_RECOVERY_RTOL = 2e-4   # sums of at most k fp32 weights, each exp2 of an fp32 log-weight (|y| of a few tens)
TOKEN_RECOVERY_ATOL = 1e-7
LSE_ATOL = 4e-3        # l sums the bf16-rounded probabilities: relative error up to 2^-9, plus fp32 exp/log


def compare_selection(ptr, idx_gpu, idx_orc, scores_orc_rows, row_meta):
    """Row by row: identical lists, or a difference made only of blocks whose oracle
    score lies within SEL_WAIVER of the oracle's threshold (score of its weakest
    admitted candidate).  Returns the number of waived rows; raises on a real mismatch.
    scores_orc_rows(r) -> (score row fp64, i)."""
    waived = 0
    for r in range(len(ptr) - 1):
        a = idx_gpu[ptr[r]:ptr[r + 1]]
        b = idx_orc[ptr[r]:ptr[r + 1]]
        if np.array_equal(a, b):
            continue
        srow, i = scores_orc_rows(r)
        assert a[0] == 0 and a[-1] == i and (np.diff(a) > 0).all(), "row %d: malformed GPU list %s" % (r, a)
        free = [j for j in b if j not in (0, i)]
        tau = min(srow[j] for j in free)
        diff = set(a.tolist()) ^ set(b.tolist())
        for j in diff:
            assert abs(srow[j] - tau) <= SEL_WAIVER, \
                "row %d %s: block %d differs, score %.9g vs threshold %.9g" % (r, row_meta(r), j, srow[j], tau)
        waived += 1
    return waived


def compare_output(out_gpu, out_orc, lse_gpu=None, lse_orc=None, tokens=None):
    """out_*: [T, H, D] fp64 (NaN in the oracle = row not computed).  Per head:
    max-abs <= OUT_MAX_ABS and max-abs / max|oracle| <= OUT_MAX_REL; lse within LSE_ATOL.
    Returns the worst errors seen: (output max-abs, output max-rel, lse max-abs)."""
    mask = ~np.isnan(out_orc)
    assert mask.any()
    worst_abs = worst_rel = 0.0
    for h in range(out_orc.shape[1]):
        m = mask[:, h, :]
        if not m.any():
            continue
        d = np.abs(out_gpu[:, h, :][m] - out_orc[:, h, :][m]).max()
        ref = np.abs(out_orc[:, h, :][m]).max()
        worst_abs = max(worst_abs, d)
        worst_rel = max(worst_rel, d / ref)
        assert d <= OUT_MAX_ABS, "head %d: max abs err %.4g" % (h, d)
        assert d / ref <= OUT_MAX_REL, "head %d: max rel err %.4g (abs %.4g / ref %.4g)" % (h, d / ref, d, ref)
    worst_lse = 0.0
    if lse_gpu is not None:
        lm = ~np.isnan(lse_orc)
        worst_lse = float(np.abs(lse_gpu[lm] - lse_orc[lm]).max())
        assert worst_lse <= LSE_ATOL, "lse max abs err %.4g" % worst_lse
    return worst_abs, worst_rel, worst_lse
