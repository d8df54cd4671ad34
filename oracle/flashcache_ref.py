"""CPU oracle for the prefill-time KV compression path (TEST INFRASTRUCTURE ONLY).

This module is the slow, plain statement of what the path computes, written
from the paper's Method section (Outlier KV Recognition Module, Eq. 5-10, and
Dynamic Budget Allocation Module, Eq. 11-12) in fp64 numpy.  It exists so that
the GPU library can be checked against something that is not itself.  Only the
tests, the smoke entry and the benchmark's cpu_baseline leg may import it; the
product path never does, and this module imports nothing from the product.

Parity pins (tests/test_oracle_*.py): scipy's orthonormal DCT-II, orthogonality
of the explicit basis, closed forms for r=1 / r=N / a single spike, Parseval,
brute-force apportionment and brute-force top-k on tiny inputs.
Parity unpinned (the paper cannot settle them; they are this build's readings):
scoring per (layer, head) with one budget per layer, the rounding of the cut-off
gamma*N to an integer, the absence of an always-keep window, and the integer
apportionment rule itself beyond its invariants.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence, Tuple

import numpy as np
import scipy.fft

# --------------------------------------------------------------------------- #
# hyper-parameters -> integers
# --------------------------------------------------------------------------- #


def cutoff_r(n_tokens: int, gamma: float) -> int:
    """Number of retained DCT modes.

    Eq. 8 keeps indices 0 <= m <= omega with omega = gamma*N, i.e. the
    floor(gamma*N)+1 lowest modes (never fewer than 1, never more than N).
    """
    r = int(math.floor(float(gamma) * n_tokens)) + 1
    return max(1, min(int(n_tokens), r))


def total_budget(layers: int, n_tokens: int, rho: float) -> int:
    """Global budget in rows per head, summed over layers: floor(rho*L*N) in [L, L*N]."""
    t = int(math.floor(float(rho) * layers * n_tokens))
    return max(layers, min(layers * n_tokens, t))


# --------------------------------------------------------------------------- #
# storage -> fp64 (exact widening)
# --------------------------------------------------------------------------- #


def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored tensor (float32 array, or uint16 bf16 bit patterns) -> float64, exactly."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        bits = np.ascontiguousarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------- #
# Eq. 6-9: orthonormal DCT-II basis, low-pass, reconstruction
# --------------------------------------------------------------------------- #


def dct_basis(n: int, r: int) -> np.ndarray:
    """Matrix M[i, m] = alpha[m] * phi_N(m, i) for 0 <= i < N, 0 <= m < r  (Eq. 7).

    phi_N(m, i) = cos(pi/N * m * (i + 1/2)) = cos(pi * m*(2i+1) / (2N)); the
    integer m*(2i+1) is reduced mod 4N (one full period) before the cosine is
    taken, so the argument never exceeds 2*pi.
    """
    i = np.arange(n, dtype=np.int64)[:, None]
    m = np.arange(r, dtype=np.int64)[None, :]
    k = (m * (2 * i + 1)) % (4 * n)
    phi = np.cos(np.pi * k.astype(np.float64) / (2.0 * n))
    alpha = np.full(r, math.sqrt(2.0 / n))
    alpha[0] = math.sqrt(1.0 / n)
    return phi * alpha[None, :]


def base_definition(x: np.ndarray, r: int) -> np.ndarray:
    """Base signal of x [N, d] by the explicit sums of Eq. 6, 8, 9.

    C[m] = alpha[m] * sum_i x[i] * phi(m, i) for m < r (coefficients above the
    cut-off are zeroed, Eq. 8); base[t] = sum_{j<r} alpha[j] * C[j] * phi(j, t).
    """
    n = x.shape[0]
    basis = dct_basis(n, r)          # [N, r]
    coeff = basis.T @ x              # Eq. 6, retained rows only
    return basis @ coeff             # Eq. 9


def base_fast(x: np.ndarray, r: int, workers: Optional[int] = None) -> np.ndarray:
    """Same result through the library's orthonormal DCT-II / DCT-III pair."""
    coeff = scipy.fft.dct(x, type=2, norm="ortho", axis=0, workers=workers)
    coeff[r:] = 0.0
    return scipy.fft.idct(coeff, type=2, norm="ortho", axis=0, workers=workers)


def coefficients_definition(x: np.ndarray) -> np.ndarray:
    """All N coefficient rows C[m] of x [N, d] (Eq. 6), explicit form."""
    return dct_basis(x.shape[0], x.shape[0]).T @ x


# --------------------------------------------------------------------------- #
# Eq. 10: deviation score
# --------------------------------------------------------------------------- #


def deviation(x: np.ndarray, base: np.ndarray) -> np.ndarray:
    """MSE between each row of x and the same row of base: mean over the d features."""
    diff = x - base
    return np.mean(diff * diff, axis=1)


def score_unit(k: np.ndarray, v: np.ndarray, r: int, route: str = "definition",
               workers: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Dev_k[x], Dev_v[x] for one (layer, head): K, V are [N, d] float64."""
    if route == "definition":
        kb, vb = base_definition(k, r), base_definition(v, r)
    elif route == "fast":
        kb, vb = base_fast(k, r, workers), base_fast(v, r, workers)
    else:
        raise ValueError(route)
    return deviation(k, kb), deviation(v, vb)


def score(K: np.ndarray, V: np.ndarray, dtype: str, r: int, route: str = "fast",
          workers: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Scores and energies of every unit.

    K, V: stored tensors [..., N, d] (any number of leading axes, e.g. [B, L, H]).
    Returns fp64 arrays: 'dev_k', 'dev_v', 'score' of shape [..., N] and 'energy'
    of shape [..., 4] = (Ehp_k, Ehp_v, Etot_k, Etot_v) where Ehp is the energy of
    the part removed by the low-pass (= d * sum_x Dev[x], equal by Parseval to the
    sum of |C[m]|^2 over the zeroed modes, Eq. 11-12) and Etot = ||X||_F^2.
    """
    lead = K.shape[:-2]
    n, d = K.shape[-2:]
    Kf = K.reshape((-1, n, d))
    Vf = V.reshape((-1, n, d))
    u = Kf.shape[0]
    dev_k = np.empty((u, n))
    dev_v = np.empty((u, n))
    energy = np.empty((u, 4))
    for i in range(u):
        k64 = widen(Kf[i], dtype)
        v64 = widen(Vf[i], dtype)
        dk, dv = score_unit(k64, v64, r, route, workers)
        dev_k[i], dev_v[i] = dk, dv
        energy[i] = (d * dk.sum(), d * dv.sum(), np.sum(k64 * k64), np.sum(v64 * v64))
    return {
        "dev_k": dev_k.reshape(lead + (n,)),
        "dev_v": dev_v.reshape(lead + (n,)),
        "score": (dev_k + dev_v).reshape(lead + (n,)),
        "energy": energy.reshape(lead + (4,)),
    }


def spectrum_energies(x: np.ndarray, r: int) -> Tuple[float, float]:
    """Eq. 11 as written, for one tensor x [N, d] (fp64): P[m] = |C[m]|^2 from the transform
    coefficients; returns (sum over m < r, sum over m >= r)."""
    c = scipy.fft.dct(x, type=2, norm="ortho", axis=0)
    p = np.sum(c * c, axis=1)
    return float(p[:r].sum()), float(p[r:].sum())


# --------------------------------------------------------------------------- #
# Eq. 11-12: per-layer outlier-energy ratio
# --------------------------------------------------------------------------- #


def layer_ratios(energy: np.ndarray) -> np.ndarray:
    """R^l = R_k^l + R_v^l from energy [L, H, 4].

    Energies of the heads of a layer are summed before the ratio is formed (the
    paper's K^l is the whole N x D matrix); K and V ratios are formed separately
    and added (Eq. 12).  A zero denominator gives a zero ratio.
    """
    e = np.asarray(energy, dtype=np.float64)
    out = np.zeros(e.shape[0])
    for l in range(e.shape[0]):
        hp_k = hp_v = tot_k = tot_v = 0.0
        for h in range(e.shape[1]):          # fixed ascending order
            hp_k += float(e[l, h, 0])
            hp_v += float(e[l, h, 1])
            tot_k += float(e[l, h, 2])
            tot_v += float(e[l, h, 3])
        rk = hp_k / tot_k if tot_k > 0.0 else 0.0
        rv = hp_v / tot_v if tot_v > 0.0 else 0.0
        out[l] = rk + rv
    return out


# --------------------------------------------------------------------------- #
# per-layer quotas under the global budget
# --------------------------------------------------------------------------- #


def allocate_detail(ratios: Sequence[float], total: int, b_min: int, b_max: int) -> Dict[str, object]:
    """Integer budgets b_l with sum(b_l) == total and b_min <= b_l <= b_max, plus how far the
    decisions taken on the way were from tipping over.

    The paper says only that the ratios are normalised into weights and quotas
    are handed out under the global ratio; the rule below is this build's reading.

    1. Ratios that are negative or not finite, or a ratio sum that is zero or not
       finite, make every ratio 1 (uniform split).
    2. Free set A = all layers, T' = T.  Repeat: S = sum of R_l over A (ascending
       l); share q_l = (T' * R_l) / S.  Let viol = sum over A of
       (clamp(q_l, b_min, b_max) - q_l) (ascending l).  If no share is outside
       the bounds, stop.  If viol > 0 pin the shares below b_min to b_min; if
       viol < 0 pin the shares above b_max to b_max; if viol == 0 pin both kinds.
       Pinned layers leave A and their rows leave T'.  (If S is 0, the layers
       still free all have ratio 0: give them ratio 1.)
    3. A single free layer takes T'.  Otherwise b_l = floor(q_l) and the
       T' - sum(floor(q_l)) left-over rows go one each to the largest fractional
       parts q_l - floor(q_l), ties to the lower layer.
    All arithmetic is IEEE double, evaluated exactly in the order written.

    Returned dict:
      budgets   int64 [L]
      margin    a relative perturbation size eps such that ratios R_l * (1 + e_l) with every
                |e_l| < eps give the same budgets.  Derivation: such a perturbation moves a share to
                q_l (1 + e_l) / (1 + ebar), ebar = the weighted mean of the e_k with weights q_k / T',
                |ebar| <= eps.  One share therefore moves by less than 2 eps (1 - q_l/T') q_l / (1 - eps)
                (e_l is itself part of ebar), and the difference of two shares by less than
                2 eps max(q_x, q_y) / (1 - eps).  So
                (i)   a share at distance D from a clamp bound keeps its side while
                      eps < D / (2 (1 - q_l/T') q_l + D);
                (ii)  when shares violate both bounds, viol keeps its sign while
                      eps < |viol| / (2 Q + |viol|), Q = sum of the out-of-bounds shares;
                (iii) the result of step 3 is floor(q_l + c) for any common offset c between
                      max_x (b_x - q_x) and min_y (b_y + 1 - q_y), so it survives while every
                      slack(x, y) = (b_y + 1 - q_y) - (b_x - q_x) stays positive (for a layer x that took
                      a left-over row and a layer y that did not, slack is the gap of their fractional
                      parts): safe while eps < slack / (2 max(q_x, q_y) + slack).
                margin is the smallest of all these.  A share that merely crosses an integer is NOT
                a cliff: its row moves from the floor to the left-over round (or back) and every
                budget stays as it was.
      cliff_pair   (x, y): the pair with the smallest bound (iii) - when the ratios drift, x is the
                first layer to hand one row to y - or None if fewer than two layers reach step 3
      pair_margin  that pair's bound (inf if there is none)
      cliff_kind   which decision set `margin`: "clamp", "viol", "pair" or "none"
      free_layers, shares, n_extra   the layers that reach step 3, their shares q_l (nan for pinned
                layers) and the number of left-over rows step 3 hands out
    """
    L = len(ratios)
    T = int(total)
    if not (1 <= b_min <= b_max):
        raise ValueError("need 1 <= b_min <= b_max")
    if not (L * b_min <= T <= L * b_max):
        raise ValueError("budget infeasible: need L*b_min <= T <= L*b_max")
    R = [float(x) for x in ratios]
    s_all = 0.0
    for x in R:
        s_all += x
    if not math.isfinite(s_all) or s_all <= 0.0 or any((not math.isfinite(x)) or x < 0.0 for x in R):
        R = [1.0] * L

    lo, hi = float(b_min), float(b_max)
    budgets = [0] * L
    active = list(range(L))
    t_left = T
    margin, kind = math.inf, "none"
    q: Dict[int, float] = {}

    def lower(value: float, what: str) -> None:
        nonlocal margin, kind
        if value < margin:
            margin, kind = value, what

    while active:
        S = 0.0
        for l in active:
            S += R[l]
        if S <= 0.0:                      # only zero-ratio layers are left: share evenly
            for l in active:
                R[l] = 1.0
            continue
        q = {l: (float(t_left) * R[l]) / S for l in active}
        if len(active) == 1:              # a single free layer takes what is left, whatever its ratio
            break
        viol = 0.0
        for l in active:
            clamped = lo if q[l] < lo else (hi if q[l] > hi else q[l])
            viol += clamped - q[l]
            for bound in (lo, hi):
                dist = abs(q[l] - bound)
                reach = 2.0 * (1.0 - q[l] / float(t_left)) * q[l]
                lower(dist / (reach + dist) if dist > 0.0 else 0.0, "clamp")
        under = [l for l in active if q[l] < lo]
        over = [l for l in active if q[l] > hi]
        if not under and not over:
            break
        if under and over:                # otherwise the sign of viol follows from the clamp sides
            oob = sum(q[l] for l in under + over)
            lower(abs(viol) / (2.0 * oob + abs(viol)) if viol != 0.0 else 0.0, "viol")
        pin_under = under if viol >= 0.0 else []
        pin_over = over if viol <= 0.0 else []
        for l in pin_under:
            budgets[l] = b_min
            t_left -= b_min
        for l in pin_over:
            budgets[l] = b_max
            t_left -= b_max
        pinned = set(pin_under) | set(pin_over)
        active = [l for l in active if l not in pinned]

    cliff_pair, pair_margin = None, math.inf
    free_layers, n_extra = list(active), 0
    shares = [q[l] if l in q and l in active else math.nan for l in range(L)]
    if len(active) == 1:                  # a single free layer takes what is left
        budgets[active[0]] = t_left
    elif active:
        fl = {l: int(math.floor(q[l])) for l in active}
        frac = {l: q[l] - float(fl[l]) for l in active}
        for l in active:
            budgets[l] = fl[l]
        n_extra = t_left - sum(fl.values())
        order = sorted(active, key=lambda l: (-frac[l], l))
        # 0 <= n_extra < len(active) unless rounding in q misbehaves badly; the
        # loops below still terminate and keep the bounds in that case
        left, pos = n_extra, 0
        while left > 0:
            l = order[pos % len(order)]
            if budgets[l] < b_max:
                budgets[l] += 1
                left -= 1
            pos += 1
        pos = 0
        rev = order[::-1]
        while left < 0:
            l = rev[pos % len(rev)]
            if budgets[l] > b_min:
                budgets[l] -= 1
                left += 1
            pos += 1
        # the budgets are floor(q_l + c) for any common offset c with
        #   max_x (b_x - q_x) <= c < min_y (b_y + 1 - q_y);
        # they survive a drift of the shares as long as that interval stays non-empty, i.e. while
        # slack(x, y) = (b_y + 1 - q_y) - (b_x - q_x) stays positive for every ordered pair.  For a layer
        # x that took a left-over row and a layer y that did not, slack is frac_x - frac_y.
        for x in active:
            for y in active:
                if x == y:
                    continue
                slack = (float(budgets[y] + 1) - q[y]) - (float(budgets[x]) - q[x])
                m = slack / (2.0 * max(q[x], q[y]) + slack) if slack > 0.0 else 0.0
                if m < pair_margin:
                    pair_margin, cliff_pair = m, (x, y)
        lower(pair_margin, "pair")
    assert sum(budgets) == T, (budgets, T)
    return {"budgets": np.asarray(budgets, dtype=np.int64), "margin": float(margin),
            "cliff_pair": cliff_pair, "pair_margin": float(pair_margin), "cliff_kind": kind,
            "free_layers": free_layers, "shares": np.asarray(shares), "n_extra": int(n_extra)}


def allocate(ratios: Sequence[float], total: int, b_min: int, b_max: int
             ) -> Tuple[np.ndarray, float]:
    """(budgets, margin) of allocate_detail."""
    det = allocate_detail(ratios, total, b_min, b_max)
    return det["budgets"], det["margin"]


def layer_offsets(budgets: np.ndarray, kv_heads: int) -> np.ndarray:
    """Row offsets of each layer in the packed output: off[l+1] = off[l] + H*b_l."""
    off = np.zeros(len(budgets) + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(budgets, dtype=np.int64) * kv_heads)
    return off


# --------------------------------------------------------------------------- #
# selection and gather
# --------------------------------------------------------------------------- #


def select(scores_f32: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest scores, ties to the lower index, returned ascending.

    The decision is taken on fp32 values (the type the scores are published in).
    """
    s = np.asarray(scores_f32, dtype=np.float32)
    n = s.shape[0]
    idx = np.arange(n, dtype=np.int64)
    order = np.lexsort((idx, -s.astype(np.float64)))     # score descending, index ascending
    return np.sort(order[:k]).astype(np.int32)


def layer_score(scores_f32: np.ndarray) -> np.ndarray:
    """One score per token of a layer from the heads' scores [H, N] (fp32 in, fp32 out).

    Reading Eq. 10 with the MSE over the whole D = H*d wide row gives the mean of the per-head
    scores.  The decision type is fp32: the heads are added in ascending order in fp32 and the
    sum is divided by H once.
    """
    s = np.asarray(scores_f32, dtype=np.float32)
    acc = s[0].copy()
    for h in range(1, s.shape[0]):
        acc = (acc + s[h]).astype(np.float32)
    return (acc / np.float32(s.shape[0])).astype(np.float32)


def select_gather(K: np.ndarray, V: np.ndarray, scores_f32: np.ndarray,
                  budgets: np.ndarray, shared: bool = False) -> Dict[str, np.ndarray]:
    """Packed compacted cache of one sequence.

    K, V: stored tensors [L, H, N, d]; scores_f32 [L, H, N]; budgets [L].
    Every head of layer l keeps budgets[l] rows: its own top rows, or with
    shared=True the top rows of the layer score (same tokens for every head).
    Output rows are ordered by layer, then head, then ascending token index;
    rows are bit copies.
    """
    L, H, N, d = K.shape
    off = layer_offsets(budgets, H)
    rows = int(off[-1])
    idx_out = np.empty(rows, dtype=np.int32)
    K_out = np.empty((rows, d), dtype=K.dtype)
    V_out = np.empty((rows, d), dtype=V.dtype)
    for l in range(L):
        b = int(budgets[l])
        shared_kept = select(layer_score(scores_f32[l]), b) if shared else None
        for h in range(H):
            kept = shared_kept if shared else select(scores_f32[l, h], b)
            o = int(off[l]) + h * b
            idx_out[o:o + b] = kept
            K_out[o:o + b] = K[l, h][kept]
            V_out[o:o + b] = V[l, h][kept]
    return {"idx": idx_out, "K_out": K_out, "V_out": V_out, "layer_offsets": off}


def scatter_paged(packed_rows: np.ndarray, budgets: np.ndarray, kv_heads: int,
                  block_table: np.ndarray, page_size: int, cache: np.ndarray) -> np.ndarray:
    """Places the packed rows of one sequence ([H*T, d], layer-major, then head) into a paged cache.

    Row j of unit (l, h) goes to slot j % page_size of page block_table[l, h, j // page_size];
    `cache` [num_pages, page_size, d] is updated in place and returned.  Rows whose page entry is
    missing or out of range are dropped.
    """
    off = layer_offsets(budgets, kv_heads)
    n_pages, max_pages = cache.shape[0], block_table.shape[-1]
    for l in range(len(budgets)):
        b = int(budgets[l])
        for h in range(kv_heads):
            o = int(off[l]) + h * b
            for j in range(b):
                p = j // page_size
                if p >= max_pages:
                    continue
                page = int(block_table[l, h, p])
                if 0 <= page < n_pages:
                    cache[page, j % page_size] = packed_rows[o + j]
    return cache


def decode_attention(Q: np.ndarray, K_rows: np.ndarray, V_rows: np.ndarray, dtype: str,
                     budgets: np.ndarray, kv_heads: int, scale: float) -> np.ndarray:
    """Decode-step attention of one sequence over its packed cache (Preliminary, Eq. 4), fp64.

    Q [L, Hq, d] (stored type), K_rows / V_rows [H*T, d] packed by layer, then head.  Query head g
    attends to the rows of KV head g // (Hq // H):  out = softmax(q K^T * scale) V.  A unit without
    rows gives zeros.
    """
    q64, k64, v64 = widen(Q, dtype), widen(K_rows, dtype), widen(V_rows, dtype)
    L, Hq, d = q64.shape
    group = Hq // kv_heads
    off = layer_offsets(budgets, kv_heads)
    out = np.zeros((L, Hq, d))
    for l in range(L):
        b = int(budgets[l])
        if b == 0:
            continue
        for g in range(Hq):
            o = int(off[l]) + (g // group) * b
            s = (k64[o:o + b] @ q64[l, g]) * scale
            p = np.exp(s - s.max())
            out[l, g] = (p / p.sum()) @ v64[o:o + b]
    return out


def decode_attention_paged(Q: np.ndarray, K_cache: np.ndarray, V_cache: np.ndarray, dtype: str,
                           budgets: np.ndarray, kv_heads: int, block_table: np.ndarray,
                           page_size: int, scale: float) -> np.ndarray:
    """Decode-step attention of one sequence over a paged cache (Preliminary, Eq. 4), fp64.

    K_cache / V_cache [num_pages, page_size, d]; row j of unit (l, h) sits in slot j % page_size of
    page block_table[l, h, j // page_size].  Rows whose page entry is missing or out of range are
    not attended to (they were never written); a unit without attended rows gives zeros.
    """
    q64 = widen(Q, dtype)
    L, Hq, d = q64.shape
    group = Hq // kv_heads
    n_pages, max_pages = K_cache.shape[0], block_table.shape[-1]
    out = np.zeros((L, Hq, d))
    for l in range(L):
        b = int(budgets[l])
        for h in range(kv_heads):
            where = []
            for j in range(b):
                pg = j // page_size
                if pg < max_pages and 0 <= int(block_table[l, h, pg]) < n_pages:
                    where.append((int(block_table[l, h, pg]), j % page_size))
            if not where:
                continue
            pages, slots = np.array(where).T
            k64, v64 = widen(K_cache[pages, slots], dtype), widen(V_cache[pages, slots], dtype)
            for g in range(h * group, (h + 1) * group):
                s_ = (k64 @ q64[l, g]) * scale
                p_ = np.exp(s_ - s_.max())
                out[l, g] = (p_ / p_.sum()) @ v64
    return out


# --------------------------------------------------------------------------- #
# whole path for a batch of sequences
# --------------------------------------------------------------------------- #


def compress(K: np.ndarray, V: np.ndarray, dtype: str, r: int, total: int,
             b_min: int = 1, b_max: Optional[int] = None, route: str = "fast",
             workers: Optional[int] = None, shared: bool = False) -> Dict[str, object]:
    """score -> allocate -> select+gather for K, V of shape [B, L, H, N, d]."""
    B, L, H, N, d = K.shape
    if b_max is None:
        b_max = N
    sc = score(K, V, dtype, r, route, workers)
    scores_f32 = sc["score"].astype(np.float32)           # published scores: one rounding
    out = {"score64": sc["score"], "scores": scores_f32, "energy": sc["energy"],
           "dev_k": sc["dev_k"], "dev_v": sc["dev_v"],
           "ratios": [], "budgets": [], "margin": [], "cliff": [], "layer_offsets": [],
           "idx": [], "K_out": [], "V_out": []}
    for b in range(B):
        R = layer_ratios(sc["energy"][b])
        det = allocate_detail(R, total, b_min, b_max)
        budgets, margin = det["budgets"], det["margin"]
        sg = select_gather(K[b], V[b], scores_f32[b], budgets, shared)
        out["ratios"].append(R)
        out["budgets"].append(budgets)
        out["margin"].append(margin)
        out["cliff"].append(det)
        out["layer_offsets"].append(sg["layer_offsets"])
        out["idx"].append(sg["idx"])
        out["K_out"].append(sg["K_out"])
        out["V_out"].append(sg["V_out"])
    for key in ("ratios", "budgets", "layer_offsets", "idx", "K_out", "V_out"):
        out[key] = np.stack(out[key])
    return out
