"""Parity rules between the GPU path and the CPU oracle, shared by the GPU tests and smoke().

Scores (fp32 on the GPU, fp64 in the oracle):
    |s_gpu - s_ref| <= 1e-4 * s_ref + 1e-7 * P,   P = mean_x (|K[x]|^2 + |V[x]|^2) / d of the unit
  (relative 1e-4 as the target states; the absolute floor scales with signal power because the
  fp32 error of the reconstruction is proportional to the base signal, not to the residual).
Index sets: bit-exact outside the tie band; a token is in the band if its oracle score is within
  relative 1e-5 of the oracle's k-th or (k+1)-th score (and, only when that threshold score is
  itself below 100x the absolute floor of the score tolerance, within twice that floor).
Budgets: bit-exact, or - only when the oracle reports two layers within relative 1e-5 of trading a
  row - different by exactly that one trade (check_budgets names which of the two happened).
Gathered rows: bit-exact copies of the rows the GPU selected.
"""
import numpy as np

SCORE_RTOL = 1e-4
SCORE_FLOOR = 1e-7
TIE_BAND = 1e-5


def to_torch(arr, dtype, device="cuda"):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def rows_to_numpy(t, dtype):
    import torch
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def unit_power(K64, V64):
    """P per unit for stored tensors already widened to fp64, shape [..., N, d] -> [...]."""
    d = K64.shape[-1]
    return (np.sum(K64 * K64, axis=-1) + np.sum(V64 * V64, axis=-1)).mean(axis=-1) / d


def check_scores(s_gpu, s_ref, power):
    """s_gpu [..., N] float32, s_ref [..., N] float64, power [...]; returns worst ratio err/tol."""
    tol = SCORE_RTOL * np.abs(s_ref) + SCORE_FLOOR * power[..., None]
    err = np.abs(s_gpu.astype(np.float64) - s_ref)
    worst = float(np.max(err / tol))
    assert worst <= 1.0, f"score error {worst:.3g} x tolerance"
    return worst


def check_index_set(idx_gpu, s_ref, k, power=None):
    """One unit: idx_gpu int32 [k] (ascending), s_ref oracle scores (fp32 values) [N].

    `power` (the unit's P of the score tolerance) only matters in the degenerate regime where the
    threshold score itself is rounding noise (the low-pass keeps nearly everything): there scores
    within the score tolerance's absolute floor of the threshold count as tied as well."""
    n = s_ref.shape[0]
    idx_gpu = np.asarray(idx_gpu)
    assert idx_gpu.shape[0] == k
    if k == 0:
        return 0
    assert idx_gpu.min() >= 0 and idx_gpu.max() < n
    assert np.all(np.diff(idx_gpu) > 0), "indices must be strictly ascending"
    s = s_ref.astype(np.float64)
    order = np.lexsort((np.arange(n), -s))
    ref_kept = np.zeros(n, dtype=bool)
    ref_kept[order[:k]] = True
    gpu_kept = np.zeros(n, dtype=bool)
    gpu_kept[idx_gpu] = True
    if k == n:
        assert gpu_kept.all()
        return 0
    tau_hi, tau_lo = s[order[k - 1]], s[order[k]]
    band = (np.abs(s - tau_hi) <= TIE_BAND * tau_hi) | (np.abs(s - tau_lo) <= TIE_BAND * tau_lo)
    if power is not None and tau_hi <= 100.0 * SCORE_FLOOR * power:
        floor = 2.0 * SCORE_FLOOR * power
        band |= (np.abs(s - tau_hi) <= floor) | (np.abs(s - tau_lo) <= floor)
    missing = ref_kept & ~gpu_kept & ~band
    extra = gpu_kept & ~ref_kept & ~band
    assert not missing.any(), f"{missing.sum()} oracle-kept tokens outside the tie band were dropped"
    assert not extra.any(), f"{extra.sum()} tokens outside the tie band were kept in error"
    return int((gpu_kept != ref_kept).sum())


def check_budgets(b_gpu, detail, total):
    """Budgets of one sequence against the oracle's allocation `detail` (oracle.allocate_detail).

    Equal, or - only if the oracle reports that two layers sit within relative TIE_BAND of trading
    a row (detail["pair_margin"]) - different by exactly that trade: one row less on the first layer
    of detail["cliff_pair"], one more on the second, everything else equal.  Returns "exact" or
    "swap x->y"."""
    b_gpu = np.asarray(b_gpu, dtype=np.int64)
    b_ref = np.asarray(detail["budgets"], dtype=np.int64)
    assert int(b_gpu.sum()) == total
    if np.array_equal(b_gpu, b_ref):
        return "exact"
    pair, pm = detail["cliff_pair"], detail["pair_margin"]
    assert pair is not None and pm <= TIE_BAND, (b_gpu, b_ref, detail["margin"], pair, pm)
    want = np.zeros_like(b_ref)
    want[pair[0]], want[pair[1]] = -1, 1
    assert np.array_equal(b_gpu - b_ref, want), (b_gpu, b_ref, pair, pm)
    return f"swap {pair[0]}->{pair[1]}"
