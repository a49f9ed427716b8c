"""Pins for the CPU oracle: each part is checked against something other than itself.

Library routines (numpy bincount / lexsort / fp64 matmul, scipy logsumexp, torch's
bf16 widening), brute force from the definition on tiny inputs, closed forms and
invariants.  A dropped term, a wrong sign or index, or a transposed operand in
oracle/vt_oracle.c fails at least one test here.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2506_22694_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Alg. 1
def test_count_equals_library_bincount():
    ids = synth.zipf_ids(50_000, 997, 1.1, seed=11, permute=True)
    c, inv = oracle.count(ids, 997)
    assert inv == 0
    assert np.array_equal(c, np.bincount(ids, minlength=997))
    assert c.sum() == ids.size


def test_count_brute_force_each_bin():
    ids = synth.zipf_ids(3000, 37, 1.1, seed=12, permute=False)
    c, _ = oracle.count(ids, 37)
    for t in range(37):
        assert c[t] == int((ids == t).sum())


def test_count_invalid_ids_are_skipped_and_tallied():
    ids = np.array([0, 5, -1, 7, 8, 7, 100, 7, -5, 2**31 - 1], dtype=np.int32)
    c, inv = oracle.count(ids, 8)
    assert inv == 5
    assert c.tolist() == [1, 0, 0, 0, 0, 1, 0, 3]
    assert c.sum() + inv == ids.size
    ids64 = np.array([3, 2**40, -2**40, 3], dtype=np.int64)
    c, inv = oracle.count(ids64, 4)
    assert inv == 2 and c.tolist() == [0, 0, 0, 2]


def test_count_chunking_and_permutation_invariance():
    ids = synth.zipf_ids(20_000, 500, 1.1, seed=13, permute=True, dtype=np.int64)
    whole, _ = oracle.count(ids, 500)
    acc, _ = oracle.count(ids[:7001], 500)
    acc, _ = oracle.count(ids[7001:], 500, counts=acc)
    assert np.array_equal(whole, acc)
    shuffled = np.random.default_rng(0).permutation(ids)
    assert np.array_equal(whole, oracle.count(shuffled, 500)[0])


def test_count_empty_stream():
    c, inv = oracle.count(np.empty(0, dtype=np.int32), 16)
    assert inv == 0 and not c.any()


# ---------------------------------------------------------------- Eq. 1, Top-K
def _selected_by_definition(counts, k):
    """id is selected iff fewer than k ids precede it in (count desc, id asc)."""
    V = len(counts)
    out = []
    for a in range(V):
        before = sum(1 for b in range(V)
                     if counts[b] > counts[a] or (counts[b] == counts[a] and b < a))
        if before < k:
            out.append(a)
    return out


def test_select_brute_force_tiny_all_k():
    rng = np.random.default_rng(21)
    cases = [np.zeros(7, dtype=np.int64), np.arange(9, dtype=np.int64), np.arange(9, dtype=np.int64)[::-1].copy(),
             np.full(6, 5, dtype=np.int64)]
    for _ in range(40):
        V = int(rng.integers(1, 13))
        cases.append(rng.integers(0, 4, size=V).astype(np.int64))   # many ties
        cases.append(rng.integers(0, 10**12, size=V).astype(np.int64))  # needs 64-bit compares
    for c in cases:
        for k in range(1, len(c) + 1):
            assert oracle.select(c, k).tolist() == _selected_by_definition(c.tolist(), k)


def test_select_matches_library_lexsort_and_invariants():
    ids = synth.zipf_ids(300_000, 5000, 1.1, seed=22, permute=True)
    c = np.bincount(ids, minlength=5000).astype(np.int64)
    order = np.lexsort((np.arange(5000), -c))          # count desc, then id asc
    prev = None
    for k in (1, 2, 17, 1024, 2500, 4999, 5000):
        m, ro = oracle.select(c, k, return_rank_order=True)
        assert np.array_equal(ro, order[:k])
        assert np.array_equal(m, np.sort(order[:k]))
        assert np.all(np.diff(m) > 0)
        sel = np.zeros(5000, dtype=bool)
        sel[m] = True
        if k < 5000:
            T = c[sel].min()
            assert T >= c[~sel].max()
            tie_sel = np.flatnonzero(sel & (c == T))
            tie_uns = np.flatnonzero(~sel & (c == T))
            if tie_sel.size and tie_uns.size:
                assert tie_sel.max() < tie_uns.min()
        if prev is not None:
            assert set(prev.tolist()) <= set(m.tolist())   # nested in k
        prev = m
    assert np.array_equal(oracle.select(c, 5000), np.arange(5000))
    top = oracle.select(c, 1)[0]
    assert top == np.flatnonzero(c == c.max())[0]


def test_select_zero_count_tail_fills_by_ascending_id():
    c = np.zeros(20, dtype=np.int64)
    c[[3, 11, 17]] = [5, 9, 5]
    assert oracle.select(c, 3).tolist() == [3, 11, 17]
    assert oracle.select(c, 6).tolist() == [0, 1, 2, 3, 11, 17]
    assert oracle.select(c, 2).tolist() == [3, 11]


# ---------------------------------------------------------------- Eq. 1, gather
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_is_row_indexing(dtype):
    W = synth.head_weights(300, 24, seed=31, dtype=dtype)
    m = np.array([0, 7, 8, 150, 299], dtype=np.int32)
    Wt = oracle.gather(W, m)
    assert Wt.dtype == W.dtype and np.array_equal(Wt, W[m])
    assert np.array_equal(oracle.gather(W, np.arange(300, dtype=np.int32)), W)


# ---------------------------------------------------------------- projection
def test_bf16_widening_matches_torch():
    import torch
    bits = np.arange(0, 65536, dtype=np.uint16)
    finite = np.isfinite(synth.bf16_bits_to_f32(bits))
    bits = bits[finite]
    # one-hot h picks W[j, 0]; the oracle's widening of every finite bf16 pattern must be torch's
    W = bits.reshape(-1, 1)
    W = np.concatenate([W, np.zeros_like(W)], axis=1)
    h = synth.f32_to_bf16_bits(np.array([[1.0, 0.0]], dtype=np.float32))
    z = oracle.logits(h, W)[0]
    ref = torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(z, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_logits_match_library_fp64_matmul(dtype):
    W = synth.head_weights(257, 96, seed=41, dtype=dtype)
    h = synth.hidden_rows(5, 96, seed=41, dtype=dtype)
    Wd = (synth.bf16_bits_to_f32(W) if dtype == "bf16" else W).astype(np.float64)
    hd = (synth.bf16_bits_to_f32(h) if dtype == "bf16" else h).astype(np.float64)
    z = oracle.logits(h, W)
    assert z.shape == (5, 257)
    ref = hd @ Wd.T
    assert np.max(np.abs(z - ref)) <= 1e-12
    # a transposed operand or a swapped index would break the asymmetric one-hot case
    e = np.zeros((2, 96), dtype=np.float32)
    e[0, 3] = 1.0
    e[1, 70] = -2.0
    eh = e if dtype == "f32" else synth.f32_to_bf16_bits(e)
    ze = oracle.logits(eh, W)
    assert np.array_equal(ze[0], Wd[:, 3]) and np.array_equal(ze[1], -2.0 * Wd[:, 70])


def test_trimmed_logits_are_full_logits_restricted_to_map():
    V, d, k = 400, 64, 90
    W = synth.head_weights(V, d, seed=42, dtype="bf16")
    h = synth.hidden_rows(3, d, seed=42, dtype="bf16")
    ids = synth.zipf_ids(5000, V, 1.1, seed=42, permute=True)
    c, _ = oracle.count(ids, V)
    m = oracle.select(c, k)
    z_full = oracle.logits(h, W)
    z_trim = oracle.logits(h, oracle.gather(W, m))
    assert np.array_equal(z_trim, z_full[:, m])
    # k = V reproduces the untrimmed head
    mV = oracle.select(c, V)
    assert np.array_equal(oracle.logits(h, oracle.gather(W, mV)), z_full)
    # renormalisation identity between the trimmed and the full softmax
    lse_f, lp_f = oracle.log_softmax(z_full)
    lse_t, lp_t = oracle.log_softmax(z_trim)
    mass = np.log(np.exp(lp_f[:, m]).sum(axis=1))
    assert np.max(np.abs(lp_t - (lp_f[:, m] - mass[:, None]))) <= 1e-12


# ---------------------------------------------------------------- log-softmax
def test_log_softmax_closed_forms():
    # h = 0: every log-prob is -ln k
    for k in (1024, 32768):
        z = np.zeros((2, k))
        lse, lp = oracle.log_softmax(z)
        assert np.allclose(lse, math.log(k), rtol=0, atol=1e-13)
        assert np.allclose(lp, -math.log(k), rtol=0, atol=1e-13)
    assert abs(-math.log(32768) - (-10.39720770839918)) < 1e-14
    assert abs(-math.log(1024) - (-6.931471805599453)) < 1e-14
    # two-level logits: a_cnt entries at value a, the rest 0
    k, a_cnt, a = 1000, 7, 3.25
    z = np.zeros((1, k))
    z[0, np.random.default_rng(5).choice(k, a_cnt, replace=False)] = a
    lse, lp = oracle.log_softmax(z)
    assert abs(lse[0] - math.log(a_cnt * math.exp(a) + k - a_cnt)) < 1e-13


def test_log_softmax_invariants_and_library():
    rng = np.random.default_rng(51)
    z = rng.normal(0, 3.0, size=(6, 777))
    z[2] += 900.0      # would overflow exp() without the max shift
    z[3] -= 900.0
    lse, lp = oracle.log_softmax(z)
    assert np.max(np.abs(lse - scipy.special.logsumexp(z, axis=1))) <= 1e-12 * 900
    assert np.max(np.abs(np.exp(lp).sum(axis=1) - 1.0)) <= 1e-12
    assert np.all(lp <= 0.0) and np.all(lse >= z.max(axis=1))
    lse2, lp2 = oracle.log_softmax(z + 12.5)
    assert np.max(np.abs(lp2 - lp)) <= 1e-11
    assert np.array_equal(oracle.lse_only(z), lse)
    # the shift must be the row maximum: any other shift overflows or underflows here
    wide = np.linspace(-1000.0, 1000.0, 401)[None, :]
    lse_w, lp_w = oracle.log_softmax(wide)
    assert np.isfinite(lse_w[0]) and abs(lse_w[0] - scipy.special.logsumexp(wide[0])) <= 1e-9
    assert lp_w[0, -1] > -0.01 and np.isfinite(lp_w).all()


# ---------------------------------------------------------------- top-m + remap
def test_top_m_brute_force_tiny_with_ties():
    rng = np.random.default_rng(61)
    for _ in range(30):
        k = int(rng.integers(1, 9))
        z = rng.integers(0, 3, size=(2, k)).astype(np.float64)        # many exact ties
        map_ = np.sort(rng.choice(50, size=k, replace=False)).astype(np.int32)
        if rng.random() < 0.5:
            map_ = map_[::-1].copy()   # ties must follow the target id, not the trimmed index
        lse = oracle.lse_only(z)
        for m in range(1, k + 1):
            ids, lp, ti = oracle.top_m(z, lse, map_, m)
            for i in range(2):
                best = sorted(range(k), key=lambda j: (-z[i, j], map_[j]))[:m]
                assert ti[i].tolist() == best
                assert ids[i].tolist() == [int(map_[j]) for j in best]
                assert np.array_equal(lp[i], z[i, best] - lse[i])


def test_top_m_matches_stable_argsort_and_argmax():
    rng = np.random.default_rng(62)
    k = 5000
    z = rng.normal(size=(4, k))
    z[1, 100] = z[1, 4000] = z[1].max() + 1.0       # exact tie at the top: lower id wins
    map_ = np.sort(rng.choice(128256, size=k, replace=False)).astype(np.int32)
    lse = oracle.lse_only(z)
    ids, lp, ti = oracle.top_m(z, lse, map_, 8)
    for i in range(4):
        ref = np.argsort(-z[i], kind="stable")[:8]   # map ascending => index order is id order
        assert np.array_equal(ti[i], ref)
    assert ti[1, 0] == 100 and ti[1, 1] == 4000
    ids1, _, ti1 = oracle.top_m(z, lse, map_, 1)
    assert np.array_equal(ti1[:, 0], np.argmax(z, axis=1))
    assert np.all(np.isin(ids, map_))
    assert np.all(np.diff(lp, axis=1) <= 0)
    # m = k returns the whole row sorted
    zs = z[:1, :64].copy()
    idsk, lpk, tik = oracle.top_m(zs, oracle.lse_only(zs), map_[:64], 64)
    assert sorted(tik[0].tolist()) == list(range(64))
    assert abs(np.exp(lpk).sum() - 1.0) < 1e-12


def test_step_h_zero_picks_lowest_ids():
    W, map_ = synth.trimmed_head_direct(300, 32, seed=63, dtype="bf16")
    h = np.zeros((2, 32), dtype=np.uint16)
    r = oracle.draft_head_step(h, W, map_, 4)
    assert np.array_equal(r["ids"], np.tile(map_[:4], (2, 1)))
    assert np.allclose(r["logp"], -math.log(300), atol=1e-13, rtol=0)


def test_step_duplicate_rows_tie_to_lower_id():
    W, map_ = synth.trimmed_head_direct(200, 64, seed=64, dtype="f32")
    h = synth.hidden_rows(1, 64, seed=64, dtype="f32")
    z = oracle.logits(h, W)
    j = int(np.argmax(z[0]))
    other = (j + 57) % 200
    W[other] = W[j]
    r = oracle.draft_head_step(h, W, map_, 2)
    lo, hi = sorted((j, other))
    assert r["trim_idx"][0].tolist() == [lo, hi]
    assert r["ids"][0].tolist() == [int(map_[lo]), int(map_[hi])]
    assert r["logp"][0, 0] == r["logp"][0, 1]


# ---------------------------------------------------------------- the paper's printed sizes
def test_head_sizes_printed_by_the_paper():
    rows = []
    with open(os.path.join(GOLDEN, "head_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                p = line.split()
                rows.append((p[0], float(p[1]), int(p[2]), int(p[3])))
    full = {r[0]: r for r in rows if r[2] > 0}
    for name, (_, printed, V, d) in full.items():
        assert round(V * d / 1e6, 1) == printed, name
    # the three Llama-3-shaped workloads use exactly these heads
    assert (synth.WORKLOADS["llama3b"].V, synth.WORKLOADS["llama3b"].d) == (128256, 3072)
    assert (synth.WORKLOADS["llama8b"].V, synth.WORKLOADS["llama8b"].d) == (128256, 4096)
    for r in rows:
        if r[2] == 0:
            k = r[1] * 1e6 / r[3]
            assert 32_000 < k < 34_000      # the paper's "32K" trimmed vocabulary
    # bytes streamed per draft step at the spec shape (bf16): k * d * 2
    assert 32768 * 3072 * 2 == 201_326_592


# ---------------------------------------------------------------- the synthetic recipe itself
def test_zipf_generator_statistics():
    wl = synth.WORKLOADS["tiny"]
    ids = synth.zipf_ids(wl.n_ids, wl.V, wl.zipf_s, wl.seed, wl.permute)
    assert ids.dtype == np.int32 and ids.min() >= 0 and ids.max() < wl.V
    c = np.bincount(ids, minlength=wl.V)
    p = np.arange(1, wl.V + 1, dtype=np.float64) ** -1.1
    p /= p.sum()
    assert abs(c[0] / wl.n_ids - p[0]) < 0.005          # top id holds about 16 %
    assert np.array_equal(ids, synth.zipf_ids(wl.n_ids, wl.V, wl.zipf_s, wl.seed, wl.permute))


def test_bf16_rounding_is_nearest_even():
    import torch
    x = np.random.default_rng(71).normal(size=10000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-40]   # exact halves -> even; a subnormal
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.f32_to_bf16_bits(x), ref)
    assert np.array_equal(synth.bf16_bits_to_f32(ref),
                          torch.from_numpy(ref.view(np.int16)).view(torch.bfloat16).float().numpy())


# ----------------------------------------------------------------------------- draft-tree selection (Sec. 4.1)
def _brute_topk(scores, K):
    """K rounds of 'take the best remaining': no sort, no key function."""
    left = list(range(len(scores)))
    out = []
    for _ in range(K):
        best = left[0]
        for c in left[1:]:
            if scores[c] > scores[best]:      # strict: the earlier index keeps a tie
                best = c
        out.append(best)
        left.remove(best)
    return out


def test_tree_expand_matches_round_by_round_extraction():
    rng = np.random.default_rng(11)
    for (n, m, K) in ((1, 1, 1), (8, 8, 8), (3, 5, 15), (16, 4, 7)):
        cum = rng.normal(-3, 1, size=n).astype(np.float32)
        lp = -np.abs(rng.normal(0, 2, size=(n, m))).astype(np.float32)
        ids = rng.integers(0, 128256, size=(n, m)).astype(np.int32)
        parent, token, score = oracle.tree_expand(cum, lp, ids, K)
        flat = [np.float32(cum[c // m]) + np.float32(lp[c // m, c % m]) for c in range(n * m)]
        want = _brute_topk(flat, K)
        assert parent.tolist() == [c // m for c in want]
        assert token.tolist() == [int(ids[c // m, c % m]) for c in want]
        assert score.tolist() == [float(flat[c]) for c in want]
        assert all(score[r] >= score[r + 1] for r in range(K - 1))


def test_tree_expand_worked_example_and_ties():
    # two frontier nodes, three children each; by hand: scores
    #   node 0: -1.0 + (-0.5, -1.5, -3.0) = -1.5, -2.5, -4.0
    #   node 1: -2.0 + (-0.5, -0.5, -2.5) = -2.5, -2.5, -4.5
    cum = np.array([-1.0, -2.0], dtype=np.float32)
    lp = np.array([[-0.5, -1.5, -3.0], [-0.5, -0.5, -2.5]], dtype=np.float32)
    ids = np.array([[10, 11, 12], [20, 21, 22]], dtype=np.int32)
    parent, token, score = oracle.tree_expand(cum, lp, ids, 4)
    # three candidates tie at -2.5: flat indices 1, 3, 4 in that order
    assert parent.tolist() == [0, 0, 1, 1] and token.tolist() == [10, 11, 20, 21]
    assert score.tolist() == [-1.5, -2.5, -2.5, -2.5]
    # signed zeros compare equal: the lower index wins
    p2, t2, _ = oracle.tree_expand(np.array([0.0], dtype=np.float32), np.array([[-0.0, 0.0]], dtype=np.float32),
                                   np.array([[7, 8]], dtype=np.int32), 1)
    assert p2.tolist() == [0] and t2.tolist() == [7]
    # the score is a single fp32 addition: 1 + 2^-24 rounds to 1 in fp32 (it would not in fp64)
    _, _, s3 = oracle.tree_expand(np.array([1.0], dtype=np.float32), np.array([[2.0 ** -24]], dtype=np.float32),
                                  np.array([[0]], dtype=np.int32), 1)
    assert s3[0] == np.float32(1.0)


def test_tree_rerank_properties():
    rng = np.random.default_rng(12)
    for (N, T) in ((1, 1), (136, 32), (392, 60), (50, 50)):
        cum = rng.normal(-5, 2, size=N).astype(np.float32)
        cum[::7] = cum[0]                      # plant ties
        idx = oracle.tree_rerank(cum, T)
        assert idx.tolist() == sorted(_brute_topk(cum.tolist(), T))
        assert np.all(np.diff(idx) > 0)
        kept = set(idx.tolist())
        worst_kept = min(cum[i] for i in kept)
        assert all(cum[i] <= worst_kept for i in range(N) if i not in kept)
    # T = N keeps everything, in index order
    assert oracle.tree_rerank(np.array([3, 1, 2], dtype=np.float32), 3).tolist() == [0, 1, 2]
    # all equal: the lowest indices
    assert oracle.tree_rerank(np.zeros(10, dtype=np.float32), 4).tolist() == [0, 1, 2, 3]


# ----------------------------------------------------------------------------- Sec. 3.2: other selection criteria
def test_rank_order_prefixes_are_the_top_k_selections():
    rng = np.random.default_rng(31)
    for V in (1, 2, 9, 40):
        for hi in (3, 10**12):
            c = rng.integers(0, hi, size=V).astype(np.int64)
            ro = oracle.rank_order(c)
            assert sorted(ro.tolist()) == list(range(V))
            for j in range(V - 1):                       # adjacent pairs obey (count desc, id asc)
                a, b = int(ro[j]), int(ro[j + 1])
                assert c[a] > c[b] or (c[a] == c[b] and a < b)
            for k in range(1, V + 1):                    # every prefix is Eq. 1's Top-K(c, k)
                assert sorted(ro[:k].tolist()) == _selected_by_definition(c.tolist(), k)
                assert np.array_equal(oracle.select(c, k, return_rank_order=True)[1], ro[:k])


def test_choose_k_worked_examples():
    c = np.array([5, 0, 50, 20, 20, 5], dtype=np.int64)          # total 100; sorted: 50 20 20 5 5 0
    assert oracle.choose_k_top_p(c, 0.5) == (1, 50, 100)
    assert oracle.choose_k_top_p(c, 0.51) == (2, 70, 100)
    assert oracle.choose_k_top_p(c, 0.9) == (3, 90, 100)
    assert oracle.choose_k_top_p(c, 0.95) == (4, 95, 100)
    assert oracle.choose_k_top_p(c, 1.0) == (5, 100, 100)        # the zero-count id is never needed
    assert oracle.choose_k_top_p(c, 0.0) == (1, 50, 100)         # k >= 1
    assert oracle.choose_k_top_p(np.zeros(4, dtype=np.int64), 0.9) == (1, 0, 0)
    assert oracle.choose_k_min_count(c, 5) == (5, 100, 100)
    assert oracle.choose_k_min_count(c, 6) == (3, 90, 100)
    assert oracle.choose_k_min_count(c, 51) == (0, 0, 100)
    assert oracle.choose_k_min_count(c, 0) == (6, 100, 100)


def test_choose_k_against_library_cumsum_and_the_stated_zipf_coverage():
    ids = synth.zipf_ids(2_000_000, 128256, 1.1, seed=2000, permute=True)
    c = np.bincount(ids, minlength=128256).astype(np.int64)
    srt = np.sort(c)[::-1]
    cs = np.cumsum(srt)
    for P in (0.1, 0.5, 0.9, 0.94, 0.999, 1.0):
        k, cov, tot = oracle.choose_k_top_p(c, P)
        assert tot == 2_000_000 and cov == cs[k - 1]
        assert cs[k - 1] >= P * tot and (k == 1 or cs[k - 2] < P * tot)
    for f in (1, 2, 14, 1000):
        k, cov, tot = oracle.choose_k_min_count(c, f)
        assert k == int((c >= f).sum()) and cov == int(c[c >= f].sum())
    # finite Zipf(1.1) over 128256 ids: the 32768 most frequent carry about 94 % of the mass
    cov32k = cs[32767] / cs[-1]
    assert 0.93 < cov32k < 0.95


def test_multi_head_step_is_the_single_head_step_row_by_row():
    # Sec. 4.1 (task-specific vocabularies): a row's result depends on its own head only
    rng = np.random.default_rng(5)
    d, m = 24, 3
    heads = []
    for k in (40, 17):
        W = rng.normal(0, 1, size=(k, d)).astype(np.float32)
        mp = np.sort(rng.choice(1000, size=k, replace=False)).astype(np.int32)
        heads.append((W, mp))
    h = rng.normal(0, 1, size=(5, d)).astype(np.float32)
    hor = [1, 0, 0, 1, 0]
    out = oracle.draft_head_step_multi(h, heads, hor, m)
    for i, j in enumerate(hor):
        one = oracle.draft_head_step(h[i:i + 1], heads[j][0], heads[j][1], m)
        assert np.array_equal(out["ids"][i], one["ids"][0])
        assert np.array_equal(out["logp"][i], one["logp"][0]) and out["lse"][i] == one["lse"][0]
        # every emitted id belongs to the row's own head, never to the other one's map alone
        assert set(out["ids"][i].tolist()) <= set(heads[j][1].tolist())
    # one head for all rows: the plain step
    same = oracle.draft_head_step_multi(h, heads, [0] * 5, m)
    plain = oracle.draft_head_step(h, heads[0][0], heads[0][1], m)
    assert np.array_equal(same["ids"], plain["ids"]) and np.array_equal(same["logp"], plain["logp"])
    # permuting the rows permutes the results
    perm = np.array([3, 0, 4, 1, 2])
    outp = oracle.draft_head_step_multi(h[perm], heads, [hor[p] for p in perm], m)
    assert np.array_equal(outp["ids"], out["ids"][perm]) and np.array_equal(outp["logp"], out["logp"][perm])
