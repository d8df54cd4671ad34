"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

Sizes here are ones the oracle finishes in seconds yet span several tiles and ragged tails.
Tolerances are the ones stated in tests/parity_util.py.
"""
import numpy as np
import pytest

import kvsynth
from kvsynth.generate import generate
from oracle import flashcache_ref as ref

import parity_util as pu

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _fc():
    import paper_2511_16786_amd as fc
    return fc


def _case(name, **kw):
    cfg = kvsynth.get_config(name)
    if kw:
        cfg = cfg.scaled(**kw)
    return cfg


CASES = {
    # name: (config, paths to test)
    "tiny": (_case("tiny"), ["dense"]),
    "tiny_ragged": (_case("tiny", n_tokens=500, kv_heads=3), ["dense"]),
    "tiny_n1": (_case("tiny", n_tokens=1, outlier_frac=0.0), ["dense"]),
    "tiny_n70_d128": (_case("tiny", n_tokens=70, head_dim=128, gamma=0.3), ["dense"]),
    "mid_small": (_case("mid", n_tokens=1024, layers=3, kv_heads=2), ["dense", "fft"]),
    "mid_half": (_case("mid", n_tokens=3072, layers=1, kv_heads=2, gamma=0.4999), ["fft"]),   # r = N/2
    "mid": (_case("mid"), ["dense", "fft"]),
    # two full low blocks in one pass (r = 2008 of N = 4096), both realisations
    "n4k_g49": (_case("mid", n_tokens=4096, layers=1, kv_heads=2, gamma=0.49), ["fft", "dense"]),
    # odd token count with a middle token (the dense path folds rows i and N-1-i)
    "odd_n777": (_case("mid", n_tokens=777, layers=2, kv_heads=2, head_dim=64, gamma=0.3), ["dense"]),
    "qwen_2l": (_case("qwen_8k", layers=2), ["fft"]),
    "long_1l": (_case("long_32k", layers=1, kv_heads=2), ["fft"]),
    "batch_16k": (_case("batch8_16k", batch=2, layers=2, kv_heads=1), ["fft"]),
    # other storage types and head dims on the fast path
    "mid_f32_d64": (_case("mid", dtype="f32", head_dim=64, n_tokens=2048, layers=2), ["fft", "dense"]),
    "mid_d24": (_case("mid", head_dim=24, n_tokens=3072, layers=1, kv_heads=2), ["fft", "dense"]),
    "mid_f32_d8": (_case("mid", dtype="f32", head_dim=8, n_tokens=2048, layers=1, gamma=0.4), ["fft", "dense"]),
    # head dims that are not multiples of 64 on the dense path (padded to 64 inside the kernels), with
    # token counts the fast path does not take
    "d40_n1000": (_case("mid", head_dim=40, n_tokens=1000, layers=2, kv_heads=2), ["dense"]),
    "d96_n777": (_case("mid", head_dim=96, n_tokens=777, layers=1, kv_heads=3, gamma=0.3), ["dense"]),
    "f32_d12_n333": (_case("mid", dtype="f32", head_dim=12, n_tokens=333, layers=2, kv_heads=1), ["dense"]),
    "d160_n1500": (_case("mid", head_dim=160, n_tokens=1500, layers=1, kv_heads=2), ["dense"]),
    # cut-offs above 2048 modes: the fast path runs several passes over an fp32 residual
    "qwen_g30": (_case("qwen_8k", layers=2, gamma=0.3), ["fft"]),
    "batch_g25": (_case("batch8_16k", batch=1, layers=1, kv_heads=2, gamma=0.25), ["fft"]),
    "long_g10": (_case("long_32k", layers=1, kv_heads=1, gamma=0.1), ["fft"]),
    # cut-offs above N/2: the fast path computes the dropped part (complement mode); one block, two
    # blocks in one pass, several passes (buffer ends as Base KV), everything kept, one 1024-block
    "qwen_g90": (_case("qwen_8k", layers=2, gamma=0.9), ["fft"]),
    "qwen_g80": (_case("qwen_8k", layers=2, kv_heads=2, gamma=0.8), ["fft"]),
    "qwen_g60": (_case("qwen_8k", layers=2, kv_heads=2, gamma=0.6), ["fft"]),
    "mid_g100": (_case("mid", n_tokens=2048, layers=2, kv_heads=2, gamma=1.0), ["fft", "dense"]),
    "mid_1k_g70_f32": (_case("mid", n_tokens=1024, layers=2, kv_heads=1, gamma=0.7, dtype="f32", head_dim=64),
                       ["fft", "dense"]),
    # token counts that are multiples of 512 or of 256 only: the fast path with a 512- or 256-point
    # register transform (more passes per cut-off), also in complement mode
    "n1536": (_case("mid", n_tokens=1536, layers=2, kv_heads=2), ["fft", "dense"]),
    "n2816_f32": (_case("mid", n_tokens=2816, layers=1, kv_heads=2, dtype="f32", head_dim=64), ["fft", "dense"]),
    "n7680_g30": (_case("qwen_8k", n_tokens=7680, n_blocks=7, layers=2, kv_heads=2, gamma=0.3), ["fft"]),
    "n7936_g85": (_case("qwen_8k", n_tokens=7936, n_blocks=7, layers=1, kv_heads=2, gamma=0.85), ["fft"]),
    "n32000": (_case("long_32k", n_tokens=32000, n_blocks=31, layers=1, kv_heads=1), ["fft"]),
    # above 32768 tokens (single exchange buffer) and a token count with an odd number of 1024-blocks
    "n64k": (_case("long_32k", n_tokens=65536, n_blocks=64, layers=1, kv_heads=1, gamma=0.02), ["fft"]),
    "n31k": (_case("long_32k", n_tokens=31744, n_blocks=30, layers=1, kv_heads=2), ["fft"]),
    "n128k": (_case("long_32k", n_tokens=131072, n_blocks=128, layers=1, kv_heads=1, gamma=0.012), ["fft"]),
    "blocks_ragged": (_case("qwen_8k", layers=2, kv_heads=2, n_tokens=3000, block_len=360), ["dense"]),
}


_cache = {}


def _inputs(case):
    if case not in _cache:
        cfg, _ = CASES[case]
        K, V = generate(cfg, workers=8)
        r = ref.cutoff_r(cfg.n_tokens, cfg.gamma)
        T = ref.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
        route = "definition" if cfg.n_tokens <= 1024 else "fast"
        out = ref.compress(K, V, cfg.dtype, r, T, route=route, workers=8)
        _cache.clear()            # keep one case resident at a time
        _cache[case] = (cfg, K, V, r, T, out)
    return _cache[case]


def _params():
    for case, (cfg, paths) in CASES.items():
        for p in paths:
            yield pytest.param(case, p, id=f"{case}-{p}")


def _supported(fc, Kt, r, path):
    desc = fc.describe(Kt)
    from paper_2511_16786_amd import binding
    return fc.resolve_path(desc, r, binding.PATHS[path]) != 0


NOISE_RATIO = 1e-4      # a layer whose high-frequency share is below this is rounding noise (Ehp ~ 1e-7 Etot)


def _compare_with_oracle(cfg, K, V, comp, out, T, seqs=None):
    """Every output of a finished Compressor run against the oracle's `out` for sequences `seqs`
    (indices into the GPU batch; `out`, K, V hold those sequences in the same order).
    Returns (worst score error / tolerance, in-band flips, budget verdict per sequence)."""
    fc = _fc()
    seqs = list(range(cfg.batch)) if seqs is None else list(seqs)
    # scores and energies
    K64, V64 = ref.widen(K, cfg.dtype), ref.widen(V, cfg.dtype)
    power = pu.unit_power(K64, V64)
    del K64, V64
    s_gpu = comp.scores[seqs].cpu().numpy()
    worst = pu.check_scores(s_gpu, out["score64"], power)
    e_gpu = comp.energy[seqs].cpu().numpy()
    assert np.allclose(e_gpu[..., 2:], out["energy"][..., 2:], rtol=1e-5)
    hp_tol = 1e-4 * out["energy"][..., :2] + 1e-7 * out["energy"][..., 2:]
    assert np.all(np.abs(e_gpu[..., :2] - out["energy"][..., :2]) <= hp_tol)
    # budgets
    b_gpu = comp.budgets[seqs].cpu().numpy()
    off_gpu = comp.layer_offsets[seqs].cpu().numpy()
    verdicts = []
    for i in range(len(seqs)):
        # the allocation stage on the energies the GPU itself produced: always bit-exact
        R_gpu = ref.layer_ratios(e_gpu[i])
        own, _ = ref.allocate(R_gpu, T, 1, cfg.n_tokens)
        assert np.array_equal(b_gpu[i], own), (b_gpu[i], own)
        # against the oracle's energies: equal, or the one trade the oracle names as on its cliff.  A
        # layer whose ratio is rounding noise (the low-pass kept everything) has no meaningful ratio
        # to compare: that layer alone enters the oracle's rule with the GPU's value
        R_ref = np.asarray(out["ratios"][i])
        noise = R_ref <= NOISE_RATIO
        det = ref.allocate_detail(np.where(noise, R_gpu, R_ref), T, 1, cfg.n_tokens) if noise.any() \
            else out["cliff"][i]
        verdicts.append(pu.check_budgets(b_gpu[i], det, T))
        assert np.array_equal(off_gpu[i], ref.layer_offsets(b_gpu[i], cfg.kv_heads))
    # index sets (against the oracle's scores, with the budgets the GPU used) and gathered rows
    idx = comp.idx[seqs].cpu().numpy()
    Ko = pu.rows_to_numpy(comp.K_out[seqs], cfg.dtype)
    Vo = pu.rows_to_numpy(comp.V_out[seqs], cfg.dtype)
    flips = 0
    cap = 2 * max(1, cfg.n_tokens // 1000)                 # in-band flips allowed per unit
    for i in range(len(seqs)):
        for l in range(cfg.layers):
            k = int(b_gpu[i, l])
            for h in range(cfg.kv_heads):
                o = int(off_gpu[i, l]) + h * k
                kept = idx[i, o:o + k]
                f = pu.check_index_set(kept, out["scores"][i, l, h], k, power[i, l, h])
                assert f <= cap or out["ratios"][i][l] <= NOISE_RATIO, f"{f} in-band flips in unit {(i, l, h)}"
                flips += f
                assert np.array_equal(Ko[i, o:o + k], K[i, l, h][kept])
                assert np.array_equal(Vo[i, o:o + k], V[i, l, h][kept])
    return worst, flips, verdicts


@pytest.mark.parametrize("case,path", list(_params()))
def test_end_to_end_matches_oracle(case, path):
    fc = _fc()
    cfg, K, V, r, T, out = _inputs(case)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    if not _supported(fc, Kt, r, path):
        pytest.skip(f"path {path} does not cover this shape")
    assert fc.cutoff_r(cfg.n_tokens, cfg.gamma) == r and fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho) == T
    comp = fc.Compressor(Kt, r, T, path=path)
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    assert fc.workspace_error(comp.workspace) == 0
    _compare_with_oracle(cfg, K, V, comp, out, T)


def _selection_properties(cfg, comp, T, K, V, seqs):
    """What must hold at any size without an oracle: budgets sum to T, indices ascending and in
    range, nothing kept scores below anything dropped (on the GPU's own scores), rows are copies."""
    b_gpu = comp.budgets.cpu().numpy()
    off = comp.layer_offsets.cpu().numpy()
    assert np.all(b_gpu.sum(axis=1) == T) and b_gpu.min() >= 1 and b_gpu.max() <= cfg.n_tokens
    for b in seqs:
        s_gpu = comp.scores[b].cpu().numpy()
        idx = comp.idx[b].cpu().numpy()
        Ko = pu.rows_to_numpy(comp.K_out[b], cfg.dtype)
        Vo = pu.rows_to_numpy(comp.V_out[b], cfg.dtype)
        assert np.array_equal(off[b], ref.layer_offsets(b_gpu[b], cfg.kv_heads))
        for l in range(cfg.layers):
            k = int(b_gpu[b, l])
            for h in range(cfg.kv_heads):
                o = int(off[b, l]) + h * k
                kept = idx[o:o + k]
                assert np.array_equal(kept, ref.select(s_gpu[l, h], k))      # exact on its own scores
                assert np.array_equal(Ko[o:o + k], K[b, l, h][kept])
                assert np.array_equal(Vo[o:o + k], V[b, l, h][kept])


@pytest.mark.parametrize("name", ["qwen_8k", "long_32k"])
def test_full_size_workload_matches_oracle(name):
    """The full 28-layer workloads in the launch configuration bench.py times, every output."""
    fc = _fc()
    cfg = kvsynth.get_config(name)
    K, V = generate(cfg, workers=16)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T, path="auto")
    assert comp.path == fc.FC_PATH_FFT
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    assert fc.workspace_error(comp.workspace) == 0
    out = ref.compress(K, V, cfg.dtype, r, T, route="fast", workers=16)
    worst, flips, verdicts = _compare_with_oracle(cfg, K, V, comp, out, T)
    print(f"{name}: worst score error {worst:.3f} of tolerance, {flips} in-band flips, budgets vs oracle "
          f"{verdicts} (oracle margin {out['margin'][0]:.3g}, pair {out['cliff'][0]['cliff_pair']}), "
          f"budgets {comp.budgets.cpu().numpy().tolist()}")
    assert all(v == "exact" or v.startswith("swap") for v in verdicts)


def test_full_size_batch8_matches_oracle_on_every_sequence():
    """Batch of 8 sequences at full size, every sequence against the oracle in full (the oracle takes
    two sequences at a time to bound host memory)."""
    fc = _fc()
    cfg = kvsynth.get_config("batch8_16k")
    K, V = generate(cfg, workers=16)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T, path="auto")
    assert comp.path == fc.FC_PATH_FFT
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    assert fc.workspace_error(comp.workspace) == 0
    del Kt, Vt
    verdicts, worst_all, flips_all = [], 0.0, 0
    for s0 in range(0, cfg.batch, 2):
        seqs = [s0, s0 + 1]
        out = ref.compress(K[seqs], V[seqs], cfg.dtype, r, T, route="fast", workers=16)
        worst, flips, v = _compare_with_oracle(cfg, K[seqs], V[seqs], comp, out, T, seqs=seqs)
        print(f"batch8_16k sequences {seqs}: worst score error {worst:.3f} of tolerance, {flips} in-band "
              f"flips, budgets vs oracle {v}, oracle margins {[f'{m:.3g}' for m in out['margin']]}", flush=True)
        verdicts += v
        worst_all, flips_all = max(worst_all, worst), flips_all + flips
        del out
    print(f"batch8_16k: {verdicts.count('exact')} of {cfg.batch} sequences have budgets bit-equal to the oracle's; "
          f"worst score error {worst_all:.3f} of tolerance; {flips_all} in-band flips")
    assert len(verdicts) == cfg.batch
    _selection_properties(cfg, comp, T, K, V, range(cfg.batch))


@pytest.mark.parametrize("L,H,N", [(1, 2, 64), (4, 4, 4096), (28, 4, 32768), (7, 3, 100)])
def test_allocate_stagewise_bit_exact(L, H, N):
    fc = _fc()
    rng = np.random.default_rng(L * 1000 + H)
    B = 5
    energy = np.empty((B, L, H, 4))
    energy[..., 2:] = rng.uniform(1.0, 100.0, (B, L, H, 2))
    energy[..., :2] = energy[..., 2:] * rng.uniform(0.0, 1.0, (B, L, H, 2)) ** 3
    energy[1] *= 1e-30                                     # tiny magnitudes
    if L > 2:
        energy[2, 0, :, :2] = 0.0                          # a layer with zero ratio
    energy[3, ..., :2] = 0.0                               # every ratio zero -> uniform
    e_t = torch.from_numpy(energy).cuda()
    cases = [(ref.total_budget(L, N, 0.2), 1, N), (L, 1, N), (L * N, 1, N)]
    if L > 1 and N >= 64:
        cases += [(ref.total_budget(L, N, 0.2), max(1, N // 8), max(1, N // 4)),
                  (ref.total_budget(L, N, 0.5), 3, int(0.6 * N))]
    for T, bmin, bmax in cases:
        budgets = torch.empty((B, L), dtype=torch.int32, device="cuda")
        offs = torch.empty((B, L + 1), dtype=torch.int64, device="cuda")
        fc.allocate(e_t, B, L, H, N, T, bmin, bmax, budgets, offs)
        bg, og = budgets.cpu().numpy(), offs.cpu().numpy()
        for b in range(B):
            want, _ = ref.allocate(ref.layer_ratios(energy[b]), T, bmin, bmax)
            assert np.array_equal(bg[b], want), (T, bmin, bmax, b, bg[b], want)
            assert np.array_equal(og[b], ref.layer_offsets(want, H))


def test_allocate_sweep_of_1000_sequences_per_launch_bit_exact():
    """Seeded apportionment sweeps, each ONE launch over 1000 sequences: the realistic 28-layer
    window, tight [b_min, b_max] windows with zero ratios and many pinned layers, and budgets that
    fill every layer to b_max - where the kernel takes its serial route for the left-over rows (a free
    layer already at b_max, or an unusual left-over count); the test shows that route was reached."""
    fc = _fc()
    rng = np.random.default_rng(77)
    B, H = 1000, 2
    sweeps = [(28, 32768, ref.total_budget(28, 32768, 0.2), 1, 32768, "wide"),
              (12, 300, 300, 3, 40, "tight"),
              (9, 64, 9 * 16, 2, 16, "full"),
              (6, 50, 6 * 20 - 1, 1, 20, "nearly full")]
    for L, N, T, bmin, bmax, kind in sweeps:
        R = rng.uniform(0.0, 1.0, (B, L)) ** rng.integers(1, 5, (B, 1))
        R[rng.uniform(size=(B, L)) < 0.1] = 0.0                      # zero ratios
        if kind in ("full", "nearly full"):
            R[::2] = rng.uniform(0.1, 1.0, (B // 2, 1))              # equal ratios: shares sit exactly on b_max
            R[::4, 0] *= 1.0 + 1e-15
        R[5] = 0.0                                                    # every ratio zero -> uniform
        # energies that give exactly these ratios: Etot = 1 per tensor and head, Ehp_k = R_l, Ehp_v = 0
        # on head 0 ... split over the heads so that the head sum is formed too
        energy = np.zeros((B, L, H, 4))
        energy[..., 2:] = 1.0
        energy[:, :, 0, 0] = R * H
        e_t = torch.from_numpy(energy).cuda()
        budgets = torch.empty((B, L), dtype=torch.int32, device="cuda")
        offs = torch.empty((B, L + 1), dtype=torch.int64, device="cuda")
        fc.allocate(e_t, B, L, H, N, T, bmin, bmax, budgets, offs)
        bg, og = budgets.cpu().numpy(), offs.cpu().numpy()
        serial = pinned = 0
        for b in range(B):
            det = ref.allocate_detail(ref.layer_ratios(energy[b]), T, bmin, bmax)
            assert np.array_equal(bg[b], det["budgets"]), (kind, b, bg[b], det["budgets"])
            assert np.array_equal(og[b], ref.layer_offsets(det["budgets"], H))
            free = det["free_layers"]
            pinned += len(free) < L
            if len(free) > 1:
                at_max = any(np.floor(det["shares"][l]) >= bmax for l in free)
                serial += at_max or not (0 <= det["n_extra"] < len(free))
        print(f"allocate sweep {kind}: L={L} T={T} [{bmin},{bmax}]: {pinned} of {B} sequences pin a layer, "
              f"{serial} take the serial left-over route; all bit-exact")
        if kind == "tight":
            assert pinned > B // 2
        if kind == "full":
            assert serial > B // 4


def _run_select(fc, K, V, dtype, scores, budgets, shared=False):
    """Stage-wise call of select_gather on given scores and budgets; returns numpy outputs."""
    B, L, H, N, d = K.shape
    Kt, Vt = pu.to_torch(K, dtype), pu.to_torch(V, dtype)
    desc = fc.describe(Kt)
    offs = np.stack([ref.layer_offsets(budgets[b], H) for b in range(B)])
    rows = int(offs[0, -1])
    assert np.all(offs[:, -1] == rows)
    s_t = torch.from_numpy(scores).cuda()
    b_t = torch.from_numpy(budgets.astype(np.int32)).cuda()
    o_t = torch.from_numpy(offs).cuda()
    idx = torch.full((B, rows), -1, dtype=torch.int32, device="cuda")
    Ko = torch.zeros((B, rows, d), dtype=Kt.dtype, device="cuda")
    Vo = torch.zeros((B, rows, d), dtype=Kt.dtype, device="cuda")
    fc.select_gather(Kt, Vt, desc, s_t, b_t, o_t, rows, idx, Ko, Vo, shared=shared)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), pu.rows_to_numpy(Ko, dtype), pu.rows_to_numpy(Vo, dtype)


@pytest.mark.parametrize("N,d,dtype", [(37, 8, "f32"), (1024, 64, "bf16"), (5000, 128, "bf16"),
                                       (32768, 128, "bf16"), (50001, 64, "bf16")])
def test_select_gather_stagewise_bit_exact_with_forced_ties(N, d, dtype):
    fc = _fc()
    rng = np.random.default_rng(N)
    B, L, H = 2, 3, 2
    if dtype == "bf16":
        K = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
        V = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
    else:
        K = rng.standard_normal((B, L, H, N, d)).astype(np.float32)
        V = rng.standard_normal((B, L, H, N, d)).astype(np.float32)
    scores = rng.gamma(2.0, 1.0, (B, L, H, N)).astype(np.float32)
    # exact ties: copy the score of 0.5 % of the tokens onto others, some across the k-th place
    n_tie = max(2, N // 200)
    for b in range(B):
        for l in range(L):
            for h in range(H):
                s = scores[b, l, h]
                src = rng.choice(N, n_tie, replace=False)
                dst = rng.choice(N, n_tie, replace=False)
                s[dst] = s[src]
                kth = np.sort(s)[::-1][max(0, N // 5 - 1)]
                s[rng.choice(N, min(N, 6), replace=False)] = kth       # pile-up right at the threshold
    scores[0, 0, 0] = 0.25                                              # one unit with all scores equal
    scores[0, 0, 1, ::3] = 0.0                                          # zeros present
    # both sequences must have the same packed row count; budgets 0, 1 and N are all exercised
    budgets = np.array([[N // 5, 1, N], [N // 5 + 1, N, 0]], dtype=np.int64)
    idx, Ko, Vo = _run_select(fc, K, V, dtype, scores, budgets)
    for b in range(B):
        want = ref.select_gather(K[b], V[b], scores[b], budgets[b])
        assert np.array_equal(idx[b], want["idx"])
        assert np.array_equal(Ko[b], want["K_out"])
        assert np.array_equal(Vo[b], want["V_out"])


@pytest.mark.parametrize("N,H", [(37, 3), (4096, 4), (32768, 4), (40000, 2)])
def test_layer_shared_selection_stagewise_bit_exact(N, H):
    """Row-wide reading of Eq. 10: one index set per layer, shared by its heads."""
    fc = _fc()
    rng = np.random.default_rng(N + H)
    B, L, d = 2, 2, 64
    K = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
    V = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
    scores = rng.gamma(2.0, 1.0, (B, L, H, N)).astype(np.float32)
    scores[0, 0, :, ::5] = 0.125                      # exact ties in the layer score
    budgets = np.array([[N // 5, N // 3], [N // 3, N // 5]], dtype=np.int64)
    idx, Ko, Vo = _run_select(fc, K, V, "bf16", scores, budgets, shared=True)
    for b in range(B):
        want = ref.select_gather(K[b], V[b], scores[b], budgets[b], shared=True)
        assert np.array_equal(idx[b], want["idx"])
        assert np.array_equal(Ko[b], want["K_out"])
        assert np.array_equal(Vo[b], want["V_out"])


def test_layer_shared_end_to_end():
    fc = _fc()
    cfg = _case("mid", n_tokens=2048, layers=3)
    K, V = generate(cfg, workers=4)
    r, T = ref.cutoff_r(2048, cfg.gamma), ref.total_budget(3, 2048, cfg.rho)
    out = ref.compress(K, V, cfg.dtype, r, T, route="fast", shared=True)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T, shared=True)
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    b_gpu = comp.budgets.cpu().numpy()
    off = comp.layer_offsets.cpu().numpy()
    idx = comp.idx.cpu().numpy()
    Ko = pu.rows_to_numpy(comp.K_out, cfg.dtype)
    pu.check_budgets(b_gpu[0], out["cliff"][0], T)
    for l in range(cfg.layers):
        k = int(b_gpu[0, l])
        ls = ref.layer_score(out["scores"][0, l])
        for h in range(cfg.kv_heads):
            o = int(off[0, l]) + h * k
            pu.check_index_set(idx[0, o:o + k], ls, k)
            assert np.array_equal(idx[0, o:o + k], idx[0, int(off[0, l]):int(off[0, l]) + k])
            assert np.array_equal(Ko[0, o:o + k], K[0, l, h][idx[0, o:o + k]])


def test_strided_layout_token_major():
    """K/V stored [B, N, L, H, d] and viewed as [B, L, H, N, d] give the same results."""
    fc = _fc()
    cfg = _case("mid", n_tokens=2048, layers=2, kv_heads=2)
    K, V = generate(cfg)
    r, T = ref.cutoff_r(2048, cfg.gamma), ref.total_budget(2, 2048, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    Kp = Kt.permute(0, 3, 1, 2, 4).contiguous().permute(0, 2, 3, 1, 4)
    Vp = Vt.permute(0, 3, 1, 2, 4).contiguous().permute(0, 2, 3, 1, 4)
    assert not Kp.is_contiguous()
    for path in ("dense", "fft"):
        a = fc.Compressor(Kt, r, T, path=path)
        a.run(Kt, Vt)
        b = fc.Compressor(Kp, r, T, path=path)
        b.run(Kp, Vp)
        torch.cuda.synchronize()
        assert torch.equal(a.scores, b.scores) and torch.equal(a.idx, b.idx)
        assert torch.equal(a.K_out, b.K_out) and torch.equal(a.V_out, b.V_out)


def test_deterministic_and_workspace_guard():
    fc = _fc()
    cfg = _case("mid", n_tokens=2048, layers=2)
    K, V = generate(cfg, workers=4)
    r, T = ref.cutoff_r(2048, cfg.gamma), ref.total_budget(2, 2048, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    for path in ("dense", "fft"):
        if not _supported(fc, Kt, r, path):
            continue
        comp = fc.Compressor(Kt, r, T, path=path)
        comp.run(Kt, Vt)
        first = [t.clone() for t in (comp.scores, comp.energy, comp.budgets, comp.idx, comp.K_out)]
        comp.run(Kt, Vt)
        torch.cuda.synchronize()
        for x, y in zip(first, (comp.scores, comp.energy, comp.budgets, comp.idx, comp.K_out)):
            assert torch.equal(x, y)
        # a workspace prepared for another cut-off is refused by the kernels, not misread
        comp.scores.fill_(-1.0)
        fc.score(Kt, Vt, comp.desc, r - 1, comp.path, comp.scores, comp.energy, comp.workspace)
        torch.cuda.synchronize()
        assert fc.workspace_error(comp.workspace) == 1
        assert bool((comp.scores == -1.0).all())


def test_hip_graph_replay_matches_eager():
    """The three calls captured into one HIP graph and replayed give the eager results every time
    (the library enqueues kernels only: no allocation, no memset node, no host synchronisation)."""
    fc = _fc()
    cfg = _case("mid", n_tokens=4096, layers=4)
    K, V = generate(cfg, workers=4)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T)
    comp.run(Kt, Vt)                                   # eager reference (also the warm-up)
    torch.cuda.synchronize()
    want = [t.clone() for t in (comp.scores, comp.energy, comp.budgets, comp.idx, comp.K_out, comp.V_out)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            comp.run(Kt, Vt)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (comp.scores, comp.idx, comp.K_out, comp.V_out):
            t.zero_()                                  # eager work between the replays
        comp.budgets.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (comp.scores, comp.energy, comp.budgets, comp.idx, comp.K_out, comp.V_out)
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"


def test_paged_gather_matches_oracle_scatter():
    """Compaction straight into a paged cache: same rows as the packed output, placed by the table."""
    fc = _fc()
    rng = np.random.default_rng(21)
    B, L, H, N, d, page = 2, 3, 2, 3000, 128, 16
    K = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
    V = rng.integers(0, 0x7F80, (B, L, H, N, d)).astype(np.uint16)
    scores = rng.gamma(2.0, 1.0, (B, L, H, N)).astype(np.float32)
    budgets = np.array([[700, 40, 1260], [1, 999, 1000]], dtype=np.int64)
    offs = np.stack([ref.layer_offsets(budgets[b], H) for b in range(B)])
    rows = int(offs[0, -1])
    max_pages = (int(budgets.max()) + page - 1) // page
    n_pages = B * L * H * max_pages + 5
    table = rng.permutation(n_pages)[:B * L * H * max_pages].reshape(B, L, H, max_pages).astype(np.int32)
    table[1, 2, 1, 3] = n_pages + 7                                   # an invalid page: its rows are dropped
    Kt, Vt = pu.to_torch(K, "bf16"), pu.to_torch(V, "bf16")
    desc = fc.describe(Kt)
    idx = torch.full((B, rows), -1, dtype=torch.int32, device="cuda")
    Kc = torch.zeros((n_pages, page, d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.zeros((n_pages, page, d), dtype=torch.bfloat16, device="cuda")
    fc.select_gather_paged(Kt, Vt, desc, torch.from_numpy(scores).cuda(),
                           torch.from_numpy(budgets.astype(np.int32)).cuda(), torch.from_numpy(offs).cuda(),
                           rows, idx, torch.from_numpy(table).cuda(), page, Kc, Vc)
    torch.cuda.synchronize()
    want_K = np.zeros((n_pages, page, d), dtype=np.uint16)
    want_V = np.zeros((n_pages, page, d), dtype=np.uint16)
    for b in range(B):
        packed = ref.select_gather(K[b], V[b], scores[b], budgets[b])
        assert np.array_equal(idx[b].cpu().numpy(), packed["idx"])
        ref.scatter_paged(packed["K_out"], budgets[b], H, table[b], page, want_K)
        ref.scatter_paged(packed["V_out"], budgets[b], H, table[b], page, want_V)
    assert np.array_equal(pu.rows_to_numpy(Kc, "bf16"), want_K)
    assert np.array_equal(pu.rows_to_numpy(Vc, "bf16"), want_V)


def test_layer_streamed_scoring_matches_oracle_and_batched():
    """Scoring layer by layer on a side stream (as prefill would hand layers over), budgets and
    selection once at the end: compared with the oracle, and bit-equal to one call over all layers."""
    fc = _fc()
    cfg = _case("mid", n_tokens=4096, layers=4)
    K, V = generate(cfg, workers=4)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T)
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    want = [t.clone() for t in (comp.scores, comp.energy, comp.idx, comp.K_out)]
    comp.scores.zero_(); comp.energy.zero_(); comp.idx.zero_(); comp.K_out.zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for l in range(cfg.layers):
            Kl, Vl = Kt[:, l:l + 1], Vt[:, l:l + 1]
            fc.score(Kl, Vl, fc.describe(Kl), r, comp.path, comp.scores[:, l:l + 1],
                     comp.energy[:, l:l + 1], comp.workspace)
        comp.run_allocate()
        comp.run_select_gather(Kt, Vt)
    side.synchronize()
    # parity proper: the layer-streamed result against the oracle ...
    out = ref.compress(K, V, cfg.dtype, r, T, route="fast", workers=8)
    _compare_with_oracle(cfg, K, V, comp, out, T)
    # ... and, as a property, bit-equality with the single call over all layers
    for a, b in zip(want, (comp.scores, comp.energy, comp.idx, comp.K_out)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("path,n", [("fft", 2048), ("dense", 700), ("fft", 8192)])
def test_layer_streamed_scoring_of_a_batch(path, n):
    """flashcache_score_layer: one call per layer covers every sequence of a batch and writes that
    layer of the full-size outputs; compared with the oracle, and bit-equal to one call over all layers."""
    fc = _fc()
    cfg = _case("mid", n_tokens=n, layers=3, kv_heads=2, batch=3, gamma=0.3 if n == 8192 else 0.1)
    K, V = generate(cfg, workers=4)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T, path=path)
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    want = [t.clone() for t in (comp.scores, comp.energy, comp.idx, comp.K_out)]
    comp.scores.fill_(-1.0); comp.energy.fill_(-1.0); comp.idx.zero_(); comp.K_out.zero_()
    # one layer of all sequences needs a workspace prepared for that shape
    K0 = Kt[:, 0:1]
    d1 = fc.describe(K0)
    ws = torch.empty(fc.workspace_bytes(d1, r, comp.path) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    fc.prepare(d1, r, comp.path, ws)
    for l in (2, 0, 1):                                      # any order
        Kl, Vl = Kt[:, l:l + 1], Vt[:, l:l + 1]
        fc.score_layer(Kl, Vl, fc.describe(Kl), l, cfg.layers, r, comp.path, comp.scores, comp.energy, ws)
    comp.run_allocate()
    comp.run_select_gather(Kt, Vt)
    torch.cuda.synchronize()
    assert fc.workspace_error(ws) == 0
    # parity proper: the layer-by-layer result against the oracle ...
    out = ref.compress(K, V, cfg.dtype, r, T, route="definition" if n <= 1024 else "fast", workers=8)
    _compare_with_oracle(cfg, K, V, comp, out, T)
    # ... and, as a property, bit-equality with the single call over all layers
    for a, b in zip(want, (comp.scores, comp.energy, comp.idx, comp.K_out)):
        assert torch.equal(a, b)


def test_layer_streamed_scoring_beside_a_producer_stream():
    """The overlap mode of bench.py at a small size: a producer stream hands layers over through
    events, flashcache_score_layer consumes them on a second stream of the same priority; the result
    must equal the batched run bit for bit (timings are printed, not asserted)."""
    import bench
    import time as _time
    fc = _fc()
    cfg = _case("qwen_8k", layers=6, n_tokens=8192)
    K, V = generate(cfg, workers=8)
    r, T = fc.cutoff_r(cfg.n_tokens, cfg.gamma), fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T)
    comp.run(Kt, Vt)
    torch.cuda.synchronize()
    bench.time = _time
    rec = bench.overlap_record(torch, fc, cfg, Kt, Vt, r, comp, reps=2, producer_mb=64)
    print(f"overlap: producer {rec['producer_alone_ms']:.2f} ms, scoring {rec['layer_scoring_alone_ms']:.2f} ms, "
          f"together {rec['together_ms']:.2f} ms")
    assert rec["scores_equal_batched_run"]


@pytest.mark.parametrize("dtype,d,Hq,H,N", [("bf16", 128, 28, 4, 4096), ("f32", 64, 4, 2, 1500),
                                           ("bf16", 128, 8, 8, 700), ("bf16", 64, 16, 2, 9000),
                                           ("bf16", 128, 12, 4, 3000), ("bf16", 64, 32, 2, 2500),
                                           ("f32", 128, 8, 1, 1000)])
def test_decode_attention_over_compacted_cache(dtype, d, Hq, H, N):
    """Decode-step attention over the ragged compacted cache against the fp64 oracle.
    Tolerance: the output is a convex combination of V rows; fp32 exp2 and accumulation over up to
    N rows leave a relative weight error of about sqrt(N)*2^-24, so |err| <= 5e-5 * max|V|."""
    fc = _fc()
    rng = np.random.default_rng(N + d)
    B, L = 2, 3
    budgets = np.array([[N // 5, 1, N // 2], [N // 2, N // 5 + 1, 0]], dtype=np.int64)
    offs = np.stack([ref.layer_offsets(budgets[b], H) for b in range(B)])
    rows = int(offs[0, -1])
    assert int(offs[1, -1]) == rows
    def make(shape, sigma=1.0):
        x = (sigma * rng.standard_normal(shape)).astype(np.float32)
        return kvsynth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    Kr, Vr, Q = make((B, rows, d)), make((B, rows, d), 2.0), make((B, L, Hq, d))
    scale = 1.0 / np.sqrt(d)
    out = fc.decode_attention(pu.to_torch(Q, dtype), pu.to_torch(Kr, dtype), pu.to_torch(Vr, dtype), H,
                              torch.from_numpy(budgets.astype(np.int32)).cuda(),
                              torch.from_numpy(offs).cuda(), rows, float(scale))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    vmax = float(np.abs(ref.widen(Vr, dtype)).max())
    for b in range(B):
        want = ref.decode_attention(Q[b], Kr[b], Vr[b], dtype, budgets[b], H, float(scale))
        err = np.abs(got[b] - want).max()
        assert err <= 5e-5 * vmax, f"decode attention error {err:.3g} (max|V| {vmax:.3g})"
    assert np.all(got[1, 2] == 0.0)                       # the layer that kept nothing


@pytest.mark.parametrize("dtype,d,Hq,H,N,page", [("bf16", 128, 28, 4, 3000, 64), ("bf16", 64, 6, 2, 1000, 17),
                                                ("f32", 64, 4, 2, 900, 32)])
def test_decode_attention_over_paged_cache(dtype, d, Hq, H, N, page):
    """Decode-step attention through a block table (pages written by the oracle's scatter) against
    the oracle; one page of one unit is unmapped, so its rows must drop out.  Same tolerance as the
    packed case."""
    fc = _fc()
    rng = np.random.default_rng(N + d + page)
    B, L = 2, 3
    budgets = np.array([[N // 4, 3, N // 2], [N // 3, 0, N // 5 + 1]], dtype=np.int64)
    offs = np.stack([ref.layer_offsets(budgets[b], H) for b in range(B)])
    rows = int(offs[:, -1].max())
    def make(shape, sigma=1.0):
        x = (sigma * rng.standard_normal(shape)).astype(np.float32)
        return kvsynth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    Kr, Vr, Q = make((B, rows, d)), make((B, rows, d), 2.0), make((B, L, Hq, d))
    max_pages = (int(budgets.max()) + page - 1) // page
    n_pages = B * L * H * max_pages + 3
    table = rng.permutation(n_pages)[:B * L * H * max_pages].reshape(B, L, H, max_pages).astype(np.int32)
    table[0, 2, 1, 1] = -1                                  # an unmapped page in the middle of a unit
    table[1, 0, 0, 0] = n_pages + 5                         # an out-of-range entry at the start of a unit
    Kc = np.zeros((n_pages, page, d), dtype=Kr.dtype)
    Vc = np.zeros((n_pages, page, d), dtype=Vr.dtype)
    for b in range(B):
        ref.scatter_paged(Kr[b], budgets[b], H, table[b], page, Kc)
        ref.scatter_paged(Vr[b], budgets[b], H, table[b], page, Vc)
    scale = 1.0 / np.sqrt(d)
    out = fc.decode_attention_paged(pu.to_torch(Q, dtype), pu.to_torch(Kc, dtype), pu.to_torch(Vc, dtype), H,
                                    torch.from_numpy(budgets.astype(np.int32)).cuda(),
                                    torch.from_numpy(table).cuda(), float(scale))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    vmax = float(np.abs(ref.widen(Vr, dtype)).max())
    for b in range(B):
        want = ref.decode_attention_paged(Q[b], Kc, Vc, dtype, budgets[b], H, table[b], page, float(scale))
        err = np.abs(got[b] - want).max()
        assert err <= 5e-5 * vmax, f"paged decode attention error {err:.3g} (max|V| {vmax:.3g})"
    assert np.all(got[1, 1] == 0.0)                        # the layer that kept nothing


@pytest.mark.parametrize("case,path", [("mid_small", "dense"), ("mid", "fft"), ("qwen_g30", "fft"),
                                       ("qwen_g80", "fft"), ("qwen_g60", "fft")])
def test_spectrum_side_energy_cross_check(case, path):
    """Eq. 11-12 as written (energies from the DCT coefficients) against the residual route."""
    fc = _fc()
    cfg, K, V, r, T, out = _inputs(case)
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    comp = fc.Compressor(Kt, r, T, path=path)
    comp.run_score(Kt, Vt)
    low = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, 2), dtype=torch.float64, device="cuda")
    fc.lowpass_energy(comp.desc, r, comp.path, comp.workspace, low)
    torch.cuda.synchronize()
    low = low.cpu().numpy()
    e = comp.energy.cpu().numpy()
    for idx in np.ndindex(cfg.batch, cfg.layers, cfg.kv_heads):
        for t, X in enumerate((K, V)):
            lo_ref, hi_ref = ref.spectrum_energies(ref.widen(X[idx], cfg.dtype), r)
            assert abs(low[idx][t] - lo_ref) <= 2e-5 * lo_ref
            # Parseval on the GPU's own numbers: total - below cut-off = above cut-off
            assert abs((e[idx][2 + t] - low[idx][t]) - e[idx][t]) <= 2e-5 * e[idx][2 + t]
            assert abs(e[idx][t] - hi_ref) <= 1e-4 * hi_ref + 1e-7 * e[idx][2 + t]


def test_random_small_shapes_against_oracle():
    """A seeded sweep of odd shapes and cut-offs (ragged N, r = 1, r = N, one layer, many heads)
    through both realisations where they apply."""
    fc = _fc()
    rng = np.random.default_rng(2024)
    shapes = []
    for _ in range(14):                                      # dense realisation: any N
        n = int(rng.choice([1, 2, 3, 31, 64, 65, 127, 200, 333, 1000, 1500]))
        shapes.append(("dense", n, int(rng.choice([64, 128])), int(rng.integers(1, n + 1))))
    shapes += [("dense", 96, 64, 96), ("dense", 257, 128, 1)]
    for _ in range(8):                                       # fast realisation: N = 1024 * n2, r <= N/2
        n = 1024 * int(rng.integers(1, 6))
        shapes.append(("fft", n, int(rng.choice([8, 16, 24, 64, 128])), int(rng.integers(1, n // 2 + 1))))
    shapes += [("fft", 2048, 128, 1), ("fft", 5120, 64, 2560)]
    for _ in range(6):                                       # ... multiples of 256 and 512 only
        n = 256 * int(rng.integers(1, 24))
        shapes.append(("fft", n, int(rng.choice([16, 64, 128])), int(rng.integers(1, n + 1))))
    for _ in range(6):                                       # ... and r > N/2 (complement mode)
        n = 1024 * int(rng.integers(1, 8))
        shapes.append(("fft", n, int(rng.choice([8, 24, 64, 128])), int(rng.integers(n // 2 + 1, n + 1))))
    shapes += [("fft", 4096, 64, 4096), ("fft", 6144, 128, 3073)]
    for path, n, d, r in shapes:
        L, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        dtype = "bf16" if rng.uniform() < 0.6 else "f32"
        cfg = _case("mid", n_tokens=n, head_dim=d, layers=L, kv_heads=H, dtype=dtype,
                    outlier_frac_range=None, outlier_frac=0.05, seed=int(rng.integers(1, 1000)))
        K, V = generate(cfg)
        T = max(L, min(L * n, int(rng.integers(L, L * n + 1))))
        out = ref.compress(K, V, dtype, r, T, route="definition" if n <= 1500 else "fast")
        Kt, Vt = pu.to_torch(K, dtype), pu.to_torch(V, dtype)
        comp = fc.Compressor(Kt, r, T, path=path)
        comp.run(Kt, Vt)
        torch.cuda.synchronize()
        assert fc.workspace_error(comp.workspace) == 0, (path, n, d, r)
        try:
            _compare_with_oracle(cfg, K, V, comp, out, T)
        except AssertionError as e:
            raise AssertionError(f"shape path={path} N={n} d={d} r={r} L={L} H={H} {dtype} T={T}: {e}")
