"""Pins for the fp64 oracle: closed forms, invariants, library routines, exact brute force.

Each test is aimed at a mistake that could plausibly be made in the oracle (a dropped
term, a wrong sign or index, a transposed operand, a wrong log base, a missing
normaliser).  None of the expected values comes from the oracle itself.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special as sps
import scipy.stats as sst

import oracle
from paper_2602_11812_amd import workloads as wl

LN2 = math.log(2.0)


def _close(a, b, atol=1e-12, rtol=0.0):
    """allclose with no relative slack unless asked for"""
    return np.allclose(a, b, rtol=rtol, atol=atol)


# ----------------------------------------------------------------------------- Eq. 2
@pytest.mark.parametrize("V", [2, 4096, 151936])
def test_entropy_uniform_is_log_v(V):
    # all logits equal => P uniform => H = ln V (natural log, not bits)
    for c in (0.0, -3.5, 1e3):
        H = oracle.entropy_from_logits(np.full((1, V), c))
        assert abs(H[0] - math.log(V)) < 1e-11


@pytest.mark.parametrize("c,expected", [(5.0, 11.927305), (12.0, 6.453048), (20.0, 6.574e-3)])
def test_entropy_one_raised_logit_printed_values(c, expected):
    # one logit c, the other V-1 at 0, V = 151936; values evaluated from the closed form
    # H = ln(e^c + V - 1) - c e^c / (e^c + V - 1)
    V = 151936
    z = np.zeros((1, V))
    z[0, 777] = c
    H = oracle.entropy_from_logits(z)[0]
    closed = math.log(math.exp(c) + V - 1) - c * math.exp(c) / (math.exp(c) + V - 1)
    assert abs(H - closed) < 1e-10
    assert abs(H - expected) < 5e-6 * max(1.0, expected) + 5e-7


def test_entropy_dominant_logit_goes_to_zero():
    V = 151936
    z = np.zeros((2, V))
    z[0, 3] = 40.0
    z[1, V - 1] = 800.0     # would overflow exp() without max subtraction
    H = oracle.entropy_from_logits(z)
    assert 0.0 <= H[0] < 1e-10
    assert H[1] == 0.0 or (0.0 <= H[1] < 1e-300)


@pytest.mark.parametrize("k,a,V", [(3, 2.0, 50), (100, -1.5, 4096), (1187, 0.25, 151936)])
def test_entropy_two_level_logits(k, a, V):
    # k logits at a, V-k at 0: H = ln Z - a k e^a / Z with Z = k e^a + V - k
    z = np.zeros((1, V))
    idx = np.random.default_rng(5).choice(V, size=k, replace=False)
    z[0, idx] = a
    Z = k * math.exp(a) + V - k
    assert abs(oracle.entropy_from_logits(z)[0] - (math.log(Z) - a * k * math.exp(a) / Z)) < 1e-10


def test_entropy_dyadic_distribution():
    # p = (1/2, 1/4, 1/8, 1/8) => H = 1.75 ln 2
    z = np.array([[-1.0, -2.0, -3.0, -3.0]]) * LN2
    assert abs(oracle.entropy_from_logits(z)[0] - 1.75 * LN2) < 1e-14
    assert abs(1.75 * LN2 - 1.2130075660) < 1e-9


def test_entropy_exact_rational_brute_force():
    # logits that are integer multiples of ln 2 give exactly rational probabilities;
    # evaluate -sum p ln p from those rationals with no exp, no max subtraction
    rng = np.random.default_rng(11)
    for _ in range(20):
        V = int(rng.integers(2, 12))
        a = rng.integers(-6, 7, size=V)
        num = [Fraction(2) ** int(x) for x in a]
        tot = sum(num)
        H_exact = -math.fsum(float(n / tot) * (math.log(n.numerator) - math.log(n.denominator)
                                                - math.log(tot.numerator) + math.log(tot.denominator))
                             for n in num)
        H = oracle.entropy_from_logits((a * LN2)[None, :])[0]
        assert abs(H - H_exact) < 1e-13


def test_entropy_matches_scipy():
    rng = np.random.default_rng(1)
    z = rng.normal(0, 3.0, size=(7, 1000))
    H = oracle.entropy_from_logits(z)
    p = sps.softmax(z, axis=1)
    assert _close(H, sps.entr(p).sum(axis=1), atol=1e-12)
    assert _close(H, sst.entropy(p, axis=1), atol=1e-12)
    # H = logsumexp(z) - E_p[z]
    assert _close(H, sps.logsumexp(z, axis=1) - (p * z).sum(axis=1), atol=1e-11)


def test_entropy_invariances():
    rng = np.random.default_rng(2)
    V = 777
    z = rng.normal(0, 2.0, size=(3, V))
    H = oracle.entropy_from_logits(z)
    assert _close(oracle.entropy_from_logits(z + 123.456), H, atol=1e-11)      # shift
    assert _close(oracle.entropy_from_logits(z[:, rng.permutation(V)]), H, atol=1e-12)
    assert _close(oracle.entropy_from_logits(np.concatenate([z, z], 1)), H + LN2, atol=1e-12)
    assert np.all(H >= 0) and np.all(H <= math.log(V))
    # sharpening (scaling logits up) never raises the entropy
    Hs = [oracle.entropy_from_logits(t * z)[0] for t in (0.0, 0.5, 1.0, 2.0, 8.0)]
    assert all(a >= b - 1e-12 for a, b in zip(Hs, Hs[1:]))
    assert abs(Hs[0] - math.log(V)) < 1e-12


def test_entropy_gaussian_logits_statistic():
    # i.i.d. N(0, s^2) logits: H ~= ln V - s^2/2 for large V
    V = 151936
    rng = np.random.default_rng(3)
    for s in (0.5, 1.0):
        H = oracle.entropy_from_logits(rng.normal(0, s, size=(1, V)))[0]
        assert abs(H - (math.log(V) - s * s / 2)) < 0.02


def test_logits_are_w_times_h_not_transposed():
    # non-square W with structured values; compare with numpy's matmul in fp64
    rng = np.random.default_rng(4)
    V, d = 37, 11
    W = rng.normal(size=(V, d)).astype(np.float32)
    h = rng.normal(size=(d,)).astype(np.float32)
    z = oracle.logits(h, W)
    assert _close(z, W.astype(np.float64) @ h.astype(np.float64), atol=1e-13)
    # a one-hot hidden state selects a column of W
    e = np.zeros(d, dtype=np.float32)
    e[3] = 1.0
    assert np.array_equal(oracle.logits(e, W), W[:, 3].astype(np.float64))


def test_entropy_through_lm_head_f32_and_bf16():
    rng = np.random.default_rng(6)
    T, V, d = 5, 301, 24
    Wf = rng.normal(0, 0.7, size=(V, d)).astype(np.float32)
    hf = rng.normal(0, 1.0, size=(T, d)).astype(np.float32)
    for W, h, Wd, hd in (
        (Wf, hf, Wf.astype(np.float64), hf.astype(np.float64)),
        (wl.to_bf16_bits(Wf), wl.to_bf16_bits(hf),
         wl.bf16_bits_to_f32(wl.to_bf16_bits(Wf)).astype(np.float64),
         wl.bf16_bits_to_f32(wl.to_bf16_bits(hf)).astype(np.float64)),
    ):
        z = hd @ Wd.T
        p = sps.softmax(z, axis=1)
        assert _close(oracle.entropy(h, W), sps.entr(p).sum(axis=1), atol=1e-11)


def test_entropy_zero_head_or_zero_hidden_gives_log_v():
    V, d = 4096, 16
    W0 = np.zeros((V, d), dtype=np.float32)
    h = np.random.default_rng(0).normal(size=(3, d)).astype(np.float32)
    assert _close(oracle.entropy(h, W0), math.log(V), atol=1e-12)
    W = np.random.default_rng(1).normal(size=(V, d)).astype(np.float32)
    assert _close(oracle.entropy(np.zeros((2, d), np.float32), W), math.log(V), atol=1e-12)


def test_bf16_rounding_of_generator_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0); 1 + 3*2^-8 ties up
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5],
                 dtype=np.float32)
    back = wl.bf16_bits_to_f32(wl.to_bf16_bits(x))
    assert back.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5]


# ----------------------------------------------------------------------------- Eq. 3, 4
def _rand_batch(seed, lens, d, dtype=np.float32):
    rng = np.random.default_rng(seed)
    T = int(sum(lens))
    hidden = rng.normal(size=(T, d)).astype(dtype)
    H = rng.uniform(0.0, 9.0, size=T)
    return hidden, H, oracle.offsets_from_lengths(lens)


def test_constant_entropy_reduces_to_mean_pooling():
    lens = [5, 1, 17, 3]
    hidden, _, off = _rand_batch(0, lens, 8)
    w, pooled, lse = oracle.pool(hidden, np.full(sum(lens), 4.2), off)
    for b, n in enumerate(lens):
        seg = hidden[off[b]:off[b + 1]].astype(np.float64)
        assert _close(pooled[b], seg.mean(axis=0), atol=1e-14)
        assert _close(w[off[b]:off[b + 1]], 1.0 / n, atol=1e-15)
        assert abs(lse[b] - (4.2 + math.log(n))) < 1e-13
    # and through the whole pipeline: a zero LM head makes every entropy ln V
    W0 = np.zeros((64, 8), dtype=np.float32)
    head = oracle.Head(w1=np.eye(8, dtype=np.float32), w2=np.ones((1, 8), np.float32))
    r = oracle.egtp(hidden, off, W0, head)
    assert _close(r.pooled, oracle.pool_ablation(hidden, off, oracle.POOL_AVERAGE), atol=1e-14)


def test_single_token_sequence_is_identity():
    hidden, H, off = _rand_batch(1, [1, 1, 1], 6)
    w, pooled, lse = oracle.pool(hidden, H, off)
    assert np.array_equal(pooled, hidden.astype(np.float64))
    assert np.array_equal(w, np.ones(3))
    assert _close(lse, H, atol=0)


def test_weights_are_softmax_of_entropy_library_and_exact():
    hidden, H, off = _rand_batch(2, [9, 4], 5)
    w, pooled, lse = oracle.pool(hidden, H, off)
    for b in range(2):
        s = slice(off[b], off[b + 1])
        assert _close(w[s], sps.softmax(H[s]), atol=1e-15)
        assert abs(lse[b] - sps.logsumexp(H[s])) < 1e-13
        # Eq. 3 exactly as printed: exp(H_i) / sum_j exp(H_j), no max subtraction
        e = [math.exp(x) for x in H[s]]
        assert _close(w[s], np.array(e) / math.fsum(e), atol=1e-15)
        # Eq. 4 with exactly summed products
        seg = hidden[s].astype(np.float64)
        for k in range(5):
            assert abs(pooled[b, k] - math.fsum(w[s] * seg[:, k])) < 1e-14
        assert abs(w[s].sum() - 1.0) < 1e-14 and np.all(w[s] > 0)
        assert np.all(pooled[b] <= seg.max(axis=0) + 1e-14) and np.all(pooled[b] >= seg.min(axis=0) - 1e-14)


def test_high_entropy_tokens_get_more_weight():
    # sign check: weight increases with entropy (exp(+H), not exp(-H))
    hidden = np.eye(3, dtype=np.float32)
    w, pooled, _ = oracle.pool(hidden, np.array([0.0, 1.0, 2.0]), [0, 3])
    assert w[0] < w[1] < w[2]
    assert _close(w[1] / w[0], math.e) and _close(pooled[0], w)


def test_ragged_indexing_constant_rows_per_sequence():
    # every token of sequence b carries the value b+1: pooled[b] must be exactly b+1,
    # whatever the entropies; an off-by-one in the offsets leaks a neighbour's value
    lens = [3, 0, 1, 7, 0, 2]
    T = sum(lens)
    off = oracle.offsets_from_lengths(lens)
    assert off.tolist() == [0, 3, 3, 4, 11, 11, 13]
    hidden = np.zeros((T, 4), dtype=np.float32)
    for b in range(len(lens)):
        hidden[off[b]:off[b + 1]] = b + 1
    H = np.random.default_rng(3).uniform(0, 12, size=T)
    w, pooled, lse = oracle.pool(hidden, H, off)
    for b, n in enumerate(lens):
        if n == 0:
            assert np.array_equal(pooled[b], np.zeros(4)) and lse[b] == -np.inf
        else:
            assert _close(pooled[b], b + 1.0, atol=1e-13)


def test_token_permutation_and_batch_composition_invariance():
    lens = [6, 11, 2]
    hidden, H, off = _rand_batch(4, lens, 7)
    _, pooled, lse = oracle.pool(hidden, H, off)
    perm = np.arange(sum(lens))
    rng = np.random.default_rng(0)
    for b in range(3):
        perm[off[b]:off[b + 1]] = rng.permutation(perm[off[b]:off[b + 1]])
    _, p2, l2 = oracle.pool(hidden[perm], H[perm], off)
    assert _close(p2, pooled, atol=1e-13) and _close(l2, lse, atol=1e-13)
    for b in range(3):        # each sequence scored alone
        s = slice(off[b], off[b + 1])
        _, p1, l1 = oracle.pool(hidden[s], H[s], [0, lens[b]])
        assert np.array_equal(p1[0], pooled[b]) and l1[0] == lse[b]


def test_temperature_limits():
    hidden, H, off = _rand_batch(5, [8], 5)
    _, hot, _ = oracle.pool(hidden, H, off, alpha=1e9)
    assert _close(hot[0], hidden.astype(np.float64).mean(axis=0), atol=1e-7)
    _, cold, _ = oracle.pool(hidden, H, off, alpha=1e-4)
    assert _close(cold[0], hidden[int(np.argmax(H))], atol=1e-12)
    w, _, _ = oracle.pool(hidden, H, off, alpha=0.5)      # this file's reading: H / alpha
    assert _close(w, sps.softmax(H / 0.5), atol=1e-15)
    with pytest.raises(ValueError):
        oracle.pool(hidden, H, off, alpha=0.0)


def test_merge_law():
    # pooling over A u B from the parts: lse = logaddexp, pooled = convex combination
    hidden, H, _ = _rand_batch(6, [23], 9)
    _, whole, lw = oracle.pool(hidden, H, [0, 23])
    for cut in (1, 7, 22):
        _, pa, la = oracle.pool(hidden[:cut], H[:cut], [0, cut])
        _, pb, lb = oracle.pool(hidden[cut:], H[cut:], [0, 23 - cut])
        l = np.logaddexp(la[0], lb[0])
        merged = pa[0] * math.exp(la[0] - l) + pb[0] * math.exp(lb[0] - l)
        assert abs(l - lw[0]) < 1e-13 and _close(merged, whole[0], atol=1e-13)


def test_pool_rejects_malformed_offsets():
    hidden, H, _ = _rand_batch(7, [4], 3)
    with pytest.raises(ValueError):
        oracle.pool(hidden, H, np.array([1, 4], dtype=np.int32))
    with pytest.raises(Exception):
        oracle.pool(hidden, H, np.array([0, 5, 4], dtype=np.int32))


def test_ablation_poolers_match_numpy():
    lens = [4, 0, 9]
    hidden, _, off = _rand_batch(8, lens, 6)
    hb = wl.to_bf16_bits(hidden)
    hd = wl.bf16_bits_to_f32(hb).astype(np.float64)
    for kind, fn in ((oracle.POOL_AVERAGE, lambda s: s.mean(0)), (oracle.POOL_MAX, lambda s: s.max(0)),
                     (oracle.POOL_LAST, lambda s: s[-1])):
        out = oracle.pool_ablation(hb, off, kind)
        for b, n in enumerate(lens):
            want = np.zeros(6) if n == 0 else fn(hd[off[b]:off[b + 1]])
            assert _close(out[b], want, atol=1e-15)


# ----------------------------------------------------------------------------- head
def _rand_head(seed, d, d_h, n_out=1, bias=True, bf16=False):
    rng = np.random.default_rng(seed)
    w1 = rng.normal(0, d ** -0.5, size=(d_h, d)).astype(np.float32)
    w2 = rng.normal(0, d_h ** -0.5, size=(n_out, d_h)).astype(np.float32)
    b1 = rng.normal(size=d_h).astype(np.float32) if bias else None
    b2 = rng.normal(size=n_out).astype(np.float32) if bias else None
    if bf16:
        w1, w2 = wl.to_bf16_bits(w1), wl.to_bf16_bits(w2)
    return oracle.Head(w1, w2, b1, b2)


def _np_head(x, head):
    def wd(a):
        return (wl.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)
    pre = x @ wd(head.w1).T + (0 if head.b1 is None else head.b1.astype(np.float64))
    return np.maximum(pre, 0) @ wd(head.w2).T + (0 if head.b2 is None else head.b2.astype(np.float64))


@pytest.mark.parametrize("bf16", [False, True])
def test_head_matches_numpy_matmul(bf16):
    x = np.random.default_rng(0).normal(size=(5, 12))
    for n_out, bias in ((1, True), (1, False), (4, True)):
        head = _rand_head(1, 12, 7, n_out, bias, bf16)
        assert _close(oracle.head_raw(x, head), _np_head(x, head), atol=1e-13)


def test_head_special_cases():
    d, d_h = 6, 5
    x = np.random.default_rng(1).normal(size=(3, d))
    head = _rand_head(2, d, d_h)
    # W1 = 0: y = b2 + w2 . relu(b1)
    z = oracle.Head(np.zeros_like(head.w1), head.w2, head.b1, head.b2)
    want = float(head.b2[0]) + float(head.w2[0].astype(np.float64) @ np.maximum(head.b1.astype(np.float64), 0))
    assert _close(oracle.predict(x, z), want, atol=1e-14)
    # all pre-activations negative: y = b2
    neg = oracle.Head(head.w1, head.w2, np.full(d_h, -1e6, np.float32), head.b2)
    assert _close(oracle.predict(x, neg), float(head.b2[0]), atol=0)
    # no biases: positively homogeneous of degree one
    nb = oracle.Head(head.w1, head.w2)
    assert _close(oracle.predict(3.5 * x, nb), 3.5 * oracle.predict(x, nb), atol=1e-13)
    # ReLU, not identity: negating the input does not negate the output in general
    assert not _close(oracle.predict(-x, nb), -oracle.predict(x, nb))


def test_bin_decode_expected_value():
    K = 20
    c = np.linspace(10.0, 1000.0, K)
    p, y = oracle.bin_decode(np.zeros((1, K)), c)
    assert _close(p, 1.0 / K) and abs(y[0] - c.mean()) < 1e-12      # uniform -> mean centre
    z = np.zeros((1, K))
    z[0, 13] = 200.0
    assert abs(oracle.bin_decode(z, c)[1][0] - c[13]) < 1e-9             # dominant bin -> its centre
    z = np.random.default_rng(0).normal(size=(4, K))
    p, y = oracle.bin_decode(z, c)
    assert _close(p, sps.softmax(z, axis=1), atol=1e-15) and _close(y, sps.softmax(z, axis=1) @ c)
    head = _rand_head(3, 8, 6, n_out=K)
    head.bin_centers = c
    x = np.random.default_rng(1).normal(size=(3, 8))
    assert _close(oracle.predict(x, head), sps.softmax(_np_head(x, head), axis=1) @ c, atol=1e-11)


# ----------------------------------------------------------------------------- plumbing
def test_tiny_config_offsets_and_seg_ids():
    w = wl.make(wl.SPECS["tiny"])
    off = oracle.offsets_from_lengths(w.lengths)
    assert off.tolist() == [0, 17, 81, 181, 309] and off.dtype == np.int32
    seg = oracle.seg_ids(off, 309)
    assert np.array_equal(seg, np.repeat(np.arange(4), [17, 64, 100, 128]))
    assert np.array_equal(seg, np.searchsorted(off, np.arange(309), side="right") - 1)
    lens = [0, 3, 0, 0, 2, 1, 0]
    off = oracle.offsets_from_lengths(lens)
    assert np.array_equal(oracle.seg_ids(off, 6), np.repeat(np.arange(7), lens))
    with pytest.raises(ValueError):
        oracle.offsets_from_lengths([3, -1])


# ----------------------------------------------------------------------------- worked example
def test_worked_example_from_eq_2_to_4_and_plp_fold():
    # Derived by hand from Eq. 2-4 (the paper prints no numeric example).  d = 2, V = 4,
    # LM-head rows (-a ln2, 0) with a = 1, 2, 3, 3, so a token (1, x) has the dyadic
    # distribution (1/2, 1/4, 1/8, 1/8), a token (0, x) the uniform one, and (200, x) is
    # one-hot to 1e-59.
    W = np.array([[-1, 0], [-2, 0], [-3, 0], [-3, 0]], dtype=np.float64) * LN2
    hidden = np.array([[0, 1], [1, 2], [200, 3]], dtype=np.float64)
    head = oracle.Head(w1=np.array([[1, -1], [0.5, 0.5]], np.float32), w2=np.array([[2, -1]], np.float32),
                       b1=np.array([0, -1], np.float32), b2=np.array([0.5], np.float32))
    r = oracle.egtp(hidden, [0, 3], W, head)
    assert _close(r.entropy, [2 * LN2, 1.75 * LN2, 0.0], atol=1e-13)
    e = np.array([4.0, 2.0 ** 1.75, 1.0])          # exp(H) = perplexities
    w = e / e.sum()
    assert _close(r.weights, w, atol=1e-14)
    assert _close(w, [0.478263768929, 0.402170288838, 0.119565942232], atol=1e-11)
    pooled = w @ hidden
    assert _close(r.pooled[0], pooled, atol=1e-12)
    assert _close(pooled, [24.315358735303, 1.641302173303], atol=1e-9)
    assert abs(r.lse[0] - math.log(e.sum())) < 1e-13 and abs(r.lse[0] - 2.123887241962) < 1e-11
    y = 0.5 + 2 * max(0.0, pooled[0] - pooled[1]) - max(0.0, 0.5 * pooled[0] + 0.5 * pooled[1] - 1)
    assert abs(r.pred[0] - y) < 1e-12 and abs(y - 33.869782669697) < 1e-8
    # PLP: fold one generated token (1, -1) with entropy 1.75 ln 2
    step = oracle.plp(hidden, [0, 3], [np.array([[1.0, -1.0]])], W, head)[0]
    e4 = np.array([4.0, 2.0 ** 1.75, 1.0, 2.0 ** 1.75])
    w4 = e4 / e4.sum()
    assert _close(step.weights, w4, atol=1e-14)
    assert _close(step.pooled[0], [17.628050758812, 0.883724248280], atol=1e-9)
    assert abs(step.lse[0] - 2.461908484567) < 1e-11 and abs(step.pred[0] - 25.732765517518) < 1e-8
    # temperature 0.5 in this file's reading (H / alpha) on the first three tokens
    w_half, p_half, _ = oracle.pool(hidden, r.entropy, [0, 3], alpha=0.5)
    assert _close(w_half, e ** 2 / (e ** 2).sum(), atol=1e-14)
    assert _close(p_half[0], [7.463300277551, 1.470221288725], atol=1e-9)


# ----------------------------------------------------------------------------- Eq. 8
def test_plp_equals_running_merge_of_prompt_state():
    # an independent streaming evaluation (numpy, merge law) of Eq. 8 must agree with the
    # oracle's recompute-from-history at every step and for every sequence
    rng = np.random.default_rng(9)
    d, V, lens, steps = 6, 50, [4, 1, 9], 5
    W = rng.normal(0, 0.8, size=(V, d)).astype(np.float32)
    prompt = rng.normal(size=(sum(lens), d)).astype(np.float32)
    gen = [rng.normal(size=(3, d)).astype(np.float32) for _ in range(steps)]
    head = _rand_head(4, d, 5)
    off = oracle.offsets_from_lengths(lens)
    res = oracle.plp(prompt, off, gen, W, head)

    def H_of(x):
        z = W.astype(np.float64) @ x.astype(np.float64)
        return float(sps.logsumexp(z) - sps.softmax(z) @ z)

    for b in range(3):
        pooled, lse = np.zeros(d), -np.inf
        toks = [prompt[i].astype(np.float64) for i in range(off[b], off[b + 1])]
        for x in toks:
            l = np.logaddexp(lse, H_of(x))
            pooled = pooled * math.exp(lse - l) + x * math.exp(H_of(x) - l)
            lse = l
        for t in range(steps):
            x = gen[t][b].astype(np.float64)
            l = np.logaddexp(lse, H_of(x))
            pooled = pooled * math.exp(lse - l) + x * math.exp(H_of(x) - l)
            lse = l
            assert _close(res[t].pooled[b], pooled, atol=1e-12)
            assert abs(res[t].lse[b] - lse) < 1e-12
            assert abs(res[t].pred[b] - _np_head(pooled[None, :], head)[0, 0]) < 1e-11


def test_tiny_config_end_to_end_against_numpy_blas():
    # the whole tiny workload against a vectorised numpy/scipy evaluation (BLAS matmul,
    # scipy softmax) as a second opinion on every stage at a realistic size
    w = wl.make(wl.SPECS["tiny"])
    off = oracle.offsets_from_lengths(w.lengths)
    head = oracle.Head(w.w1, w.w2)
    r = oracle.egtp(w.hidden, off, w.w_lm, head)
    z = w.hidden.astype(np.float64) @ w.w_lm.astype(np.float64).T
    H = sps.logsumexp(z, axis=1) - (sps.softmax(z, axis=1) * z).sum(axis=1)
    assert _close(r.entropy, H, atol=1e-11)
    for b in range(4):
        s = slice(off[b], off[b + 1])
        pooled = sps.softmax(H[s]) @ w.hidden[s].astype(np.float64)
        assert _close(r.pooled[b], pooled, atol=1e-12)
        assert abs(r.pred[b] - _np_head(pooled[None], head)[0, 0]) < 1e-12
    # entropies sit near ln V - |h|^2 / (2 d) for this generator
    approx = math.log(4096) - (w.hidden.astype(np.float64) ** 2).sum(1) / (2 * 256)
    assert np.abs(r.entropy - approx).max() < 0.1
