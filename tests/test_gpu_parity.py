"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded inputs.  Integer work is compared bit for bit; floating point to the stated bars."""
import math
import os

import numpy as np
import pytest

import oracle
from helpers import (TOL_ENTROPY_ABS, TOL_LSE_ABS, TOL_POOLED_REL_L2, assert_egtp_close, assert_pred_close, rel_l2)
from paper_2602_11812_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2602_11812_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    return binding


def _np(d):
    return {k: v.cpu().numpy() for k, v in d.items()}


def _scorer(gpu, w, alpha=1.0, b1=None, b2=None, w2=None, centers=None, head_rem=None, pack_w_lm=True):
    td = gpu.to_device
    head = gpu.make_head(td(w.w1), td(w.w2 if w2 is None else w2),
                         None if b1 is None else td(b1), None if b2 is None else td(b2),
                         None if centers is None else td(centers))
    return gpu.Scorer(td(w.w_lm), head, head_rem, alpha, pack_w_lm)


def _offsets_on_gpu(gpu, sc, lengths, want_seg=False):
    import torch
    T = int(np.sum(lengths))
    return sc.build_offsets(torch.from_numpy(np.asarray(lengths, dtype=np.int32)).cuda(), T, want_seg)


def _run(gpu, w, lengths=None, **kw):
    sc = _scorer(gpu, w, **kw)
    lengths = w.lengths if lengths is None else lengths
    off = _offsets_on_gpu(gpu, sc, lengths)
    out = _np(sc.score(gpu.to_device(w.hidden), off))
    out["offsets"] = off.cpu().numpy()
    return out


# ----------------------------------------------------------------------------- fp32 tiny workload
def test_tiny_fp32_end_to_end(gpu):
    w = wl.make(wl.SPECS["tiny"])
    got = _run(gpu, w)
    off = oracle.offsets_from_lengths(w.lengths)
    assert np.array_equal(got["offsets"], off) and got["offsets"].dtype == np.int32
    assert got["offsets"].tolist() == [0, 17, 81, 181, 309]
    want = oracle.egtp(w.hidden, off, w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)
    assert np.abs(got["entropy"] - want.entropy).max() <= 2e-5        # fp32 inputs: fp32-grade, not bf16-grade


def _fp32_case(seed, lengths, d, V):
    return wl.make(wl.scaled(wl.SPECS["tiny"], seed=seed, B=len(lengths), d=d, V=V, d_h=16, lengths=tuple(lengths)))


def test_fp32_inputs_integer_logits_are_exact(gpu):
    """fp32 operands go through the bf16 matrix cores as sums of bf16 pieces.  With 10-bit integer weights and
    11-bit integer activations (times a power of two) every piece product and every partial sum is an integer
    below 2^24, so the logits have to come out exactly, whatever the order of the additions: what is left is the
    fp32 evaluation of the softmax statistics.  Each value needs two pieces, so a lost cross product (second piece
    times second piece: a few units of 2^-12 on logits that differ by a few units) shows at once."""
    w = _fp32_case(seed=301, lengths=(130, 1, 169), d=8, V=700)
    rng = np.random.default_rng(301)
    w.w_lm = rng.integers(512, 520, size=(700, 8)).astype(np.float32)
    w.hidden = (rng.integers(1024, 2048, size=(w.T, 8)).astype(np.float32) * np.float32(2.0 ** -12))
    assert (w.w_lm.astype(np.float64) @ w.hidden.astype(np.float64).T).max() * 2 ** 12 < 2 ** 24
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2))
    assert 0.5 < want.entropy.min() and want.entropy.max() < np.log(700) - 0.01      # neither peaked nor flat
    err = np.abs(got["entropy"] - want.entropy).max()
    assert err <= 2e-5, err
    assert_egtp_close(got, want)


@pytest.mark.parametrize("side", ["w_lm", "hidden"])
def test_fp32_inputs_keep_every_mantissa_bit(gpu, side):
    """One operand is a 0/1 selection matrix, the other holds values near 1000 with full 24-bit mantissas: a
    logit is then one element of that operand, exact only if all three of its bf16 pieces arrive (the last
    piece of a value near 1000 is worth up to 0.015; the logits of a token differ by about one)."""
    n = 300
    w = _fp32_case(seed=302, lengths=(200, 100), d=n, V=n)
    rng = np.random.default_rng(302 + (side == "hidden"))
    full = (1000.0 + rng.standard_normal((n, n))).astype(np.float32)
    assert np.any(full.view(np.uint32) & 0xff)                                        # low mantissa bits in use
    eye = np.eye(n, dtype=np.float32)
    if side == "w_lm":
        w.w_lm, w.hidden = full, eye[rng.integers(0, n, size=w.T)]                   # logits of token t: a column of W_lm
    else:
        w.w_lm, w.hidden = eye, full[:w.T].copy()                                     # logits of token t: its own hidden state
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2))
    err = np.abs(got["entropy"] - want.entropy).max()
    assert err <= 2e-5, err


@pytest.mark.parametrize("case", range(6))
def test_fp32_seeded_random_shapes_against_the_oracle(gpu, case):
    """fp32 hidden states and weights at seeded shapes: hidden sizes that are multiples of 4 but (mostly) not
    of 32, so the six K segments carry zero padding; several vocabulary tiles and ragged token blocks; W_lm
    packed up front or by the call itself.  Entropies to fp32 grade, the rest at the stated bars."""
    rng = np.random.default_rng(5000 + case)
    B = int(rng.integers(1, 7))
    lens = tuple(int(x) for x in np.where(rng.random(B) < 0.15, 0, rng.integers(1, 300, size=B)))
    d = 4 * int(rng.integers(1, 90))
    V = int(rng.integers(1, 3000))
    alpha = float(rng.choice([0.5, 1.0, 2.5]))
    w = wl.make(wl.scaled(wl.SPECS["tiny"], seed=5100 + case, B=B, d=d, V=V, d_h=int(rng.integers(1, 50)),
                          lengths=lens))
    assert w.hidden.dtype == np.float32 and w.w_lm.dtype == np.float32
    got = _run(gpu, w, alpha=alpha, pack_w_lm=bool(case % 2))
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(lens), w.w_lm, oracle.Head(w.w1, w.w2), alpha)
    assert_egtp_close(got, want)
    if want.entropy.size:
        assert np.abs(got["entropy"] - want.entropy).max() <= 2e-5


def test_fp32_plp_steps_and_a_context_on_the_packed_copy_alone(gpu):
    """fp32 inputs through the decode path (one-token folds, Eq. 8) on a context that was created without the
    row-major W_lm and lives on a packed copy made by another context of the same shape."""
    import torch
    lens = (5, 40, 1, 0, 77)
    w = wl.make(wl.scaled(wl.SPECS["tiny"], seed=5200, B=len(lens), d=100, V=1300, d_h=20, lengths=lens))
    gen = [wl.decode_hidden(w.spec, t + 1) for t in range(3)]
    assert gen[0].dtype == np.float32
    td = gpu.to_device
    packer = _scorer(gpu, w)                                            # packs W_lm at creation
    head = gpu.make_head(td(w.w1), td(w.w2))
    cfg = gpu.egtp_config()
    cfg.d, cfg.vocab, cfg.dtype, cfg.w_lm, cfg.alpha, cfg.head_len = 100, 1300, gpu.EGTP_F32, None, 1.0, head
    ctx = gpu.egtp_create(cfg)
    try:
        assert gpu.egtp_packed_w_lm_bytes(ctx) == packer._w_packed.numel() == 6 * 128 * 2 * 6 * 256   # 6 row tiles x 6 segments of 128
        gpu.egtp_adopt_packed_w_lm(ctx, packer._w_packed)
        B, T = len(lens), w.T
        ws = torch.empty(gpu.egtp_workspace_bytes(ctx, T, B), dtype=torch.uint8, device="cuda")
        off = torch.from_numpy(oracle.offsets_from_lengths(lens)).cuda()
        ent = torch.empty(T, dtype=torch.float32, device="cuda")
        pooled = torch.empty(B, 100, dtype=torch.float32, device="cuda")
        lse = torch.empty(B, dtype=torch.float32, device="cuda")
        pred = torch.empty(B, dtype=torch.float32, device="cuda")
        gpu.egtp_score(ctx, td(w.hidden), off, None, B, T, ws, ent, pooled, lse, pred)
        want = oracle.plp(w.hidden, oracle.offsets_from_lengths(lens), gen, w.w_lm, oracle.Head(w.w1, w.w2))
        for t, g in enumerate(gen):
            e1 = torch.empty(B, dtype=torch.float32, device="cuda")
            gpu.plp_step(ctx, td(g), None, None, None, B, B, pooled, lse, ws, e1, pred)
            r = want[t]
            new_tok = oracle.offsets_from_lengths(np.asarray(lens) + t + 1)[1:] - 1
            assert np.abs(e1.cpu().numpy() - r.entropy[new_tok]).max() <= 2e-5
            for b in range(B):
                assert rel_l2(pooled[b].cpu().numpy(), r.pooled[b]) <= TOL_POOLED_REL_L2
            assert np.abs(lse.cpu().numpy() - r.lse).max() <= TOL_LSE_ABS
            assert_pred_close(pred.cpu().numpy(), r.pred)
    finally:
        gpu.egtp_destroy(ctx)


def test_fp32_head_small_batch_with_slots(gpu):
    """fp32 head weights and at most 16 live sequences: the first head layer streams W1 slice by slice (three
    slices of d = 2308, the last of 260 elements; d_h = 37 leaves a last group of 5 rows) and reads each
    sequence's state through its slot."""
    import torch
    lens = (3, 0, 9, 1, 30, 2, 7)
    w = wl.make(wl.scaled(wl.SPECS["tiny"], seed=5300, B=len(lens), d=2308, V=130, d_h=37, lengths=lens))
    gen = [wl.decode_hidden(w.spec, t + 1) for t in range(2)]
    sc = _scorer(gpu, w)
    B, d, S = len(lens), 2308, 11
    slot = np.array([10, 4, 0, 7, 2, 9, 5], dtype=np.int32)
    slot_dev = torch.from_numpy(slot).cuda()
    pooled = torch.zeros(S, d, dtype=torch.float32, device="cuda")
    lse = torch.full((S,), -math.inf, dtype=torch.float32, device="cuda")
    out = sc.score(gpu.to_device(w.hidden), _offsets_on_gpu(gpu, sc, lens))
    want0 = oracle.egtp(w.hidden, oracle.offsets_from_lengths(lens), w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(_np(out), want0)
    pooled[slot_dev.long()] = out["pooled"]
    lse[slot_dev.long()] = out["lse"]
    want = oracle.plp(w.hidden, oracle.offsets_from_lengths(lens), gen, w.w_lm, oracle.Head(w.w1, w.w2))
    for t, g in enumerate(gen):
        pred = sc.step(gpu.to_device(g), pooled, lse, slot_dev=slot_dev)
        r = want[t]
        for b in range(B):
            assert rel_l2(pooled[slot[b]].cpu().numpy(), r.pooled[b]) <= TOL_POOLED_REL_L2
        assert_pred_close(pred.cpu().numpy(), r.pred)
    untouched = np.setdiff1d(np.arange(S), slot)
    assert bool((pooled[torch.from_numpy(untouched).cuda()] == 0).all())


def test_offsets_and_segment_ids_bit_exact(gpu):
    w = wl.make(wl.SPECS["tiny"])
    sc = _scorer(gpu, w)
    rng = np.random.default_rng(0)
    for lens in ([17, 64, 100, 128], [0, 3, 0, 0, 2, 1, 0], [5], [0], rng.integers(0, 40, size=700).tolist(),
                 rng.integers(0, 3, size=2000).tolist()):
        T = int(np.sum(lens))
        off, seg = _offsets_on_gpu(gpu, sc, lens, want_seg=True)
        want_off = oracle.offsets_from_lengths(lens)
        assert np.array_equal(off.cpu().numpy(), want_off)
        assert np.array_equal(seg.cpu().numpy(), oracle.seg_ids(want_off, T))


# ----------------------------------------------------------------------------- bf16 matrix-core kernel
def _small_bf16(seed=1, B=6, d=512, V=2500, d_h=96, lengths=None, lo=16, hi=400):
    spec = wl.scaled(wl.SPECS["mid"], seed=seed, B=B, d=d, V=V, d_h=d_h, len_lo=lo, len_hi=hi,
                     len_mu=5.0, len_sigma=0.8, lengths=lengths)
    return wl.make(spec)


@pytest.mark.parametrize("pack_w_lm", [True, False])
def test_bf16_mfma_several_tiles_and_ragged_tails(gpu, pack_w_lm):
    # V = 2500 -> 10 vocabulary tiles, the last one ragged; T spans several 256-token blocks
    # with a ragged last block; d = 512 -> 16 K steps through the LDS ring.  W_lm is packed
    # once up front, or re-packed into the workspace by the call itself.
    w = _small_bf16()
    assert w.T > 600 and w.T % 256 != 0
    got = _run(gpu, w, pack_w_lm=pack_w_lm)
    off = oracle.offsets_from_lengths(w.lengths)
    want = oracle.egtp(w.hidden, off, w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


@pytest.mark.parametrize("T,V,d", [(1, 256, 64), (255, 257, 64), (256, 511, 128), (257, 512, 192), (513, 1000, 320),
                                   (300, 769, 96), (2, 255, 32)])
def test_bf16_mfma_edge_sizes(gpu, T, V, d):
    w = _small_bf16(seed=7, B=1, d=d, V=V, d_h=8, lengths=(T,))
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, [0, T], w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


def test_bf16_shapes_that_need_padding(gpu):
    # hidden size not a multiple of the 32-element K step, vocabulary below one 256-row tile:
    # the packed copies are zero-padded and the padded vocabulary rows masked
    for d, V in ((72, 100), (128, 200), (40, 3000), (8, 1)):
        w = _small_bf16(seed=3, B=3, d=d, V=V, d_h=16, lengths=(5, 70, 1))
        got = _run(gpu, w)
        want = oracle.egtp(w.hidden, [0, 5, 75, 76], w.w_lm, oracle.Head(w.w1, w.w2))
        assert_egtp_close(got, want)


def test_closed_forms_on_gpu(gpu):
    import torch
    # zero LM head: every entropy is ln V, pooling is the plain mean
    w = _small_bf16(seed=5, B=3, d=128, V=1187, d_h=8, lengths=(10, 1, 300))
    w.w_lm[:] = 0
    got = _run(gpu, w)
    assert np.abs(got["entropy"] - math.log(1187)).max() < 1e-5
    hf = wl.bf16_bits_to_f32(w.hidden).astype(np.float64)
    off = [0, 10, 11, 311]
    for b in range(3):
        assert rel_l2(got["pooled"][b], hf[off[b]:off[b + 1]].mean(axis=0)) < 1e-5
    assert np.allclose(got["lse"], math.log(1187) + np.log([10, 1, 300]), atol=1e-4)
    # one vocabulary row aligned with the hidden state dominates: entropy -> closed form
    V, d = 1000, 64
    W = np.zeros((V, d), dtype=np.float32)
    W[123, 0] = 4.0
    h = np.zeros((3, d), dtype=np.float32)
    h[:, 0] = [1.0, 3.0, 10.0]          # logit c = 4, 12, 40 on one row, 0 elsewhere
    w2 = wl.Workload(w.spec, np.array([3], np.int32), wl.to_bf16_bits(h), wl.to_bf16_bits(W),
                     wl.to_bf16_bits(np.ones((4, d), np.float32)), wl.to_bf16_bits(np.ones((1, 4), np.float32)))
    got = _run(gpu, w2)
    for i, c in enumerate((4.0, 12.0, 40.0)):
        Z = math.exp(c) + V - 1
        assert abs(got["entropy"][i] - (math.log(Z) - c * math.exp(c) / Z)) < 1e-4


def test_empty_and_single_token_sequences(gpu):
    lens = (0, 1, 0, 300, 1, 0)
    w = _small_bf16(seed=11, B=6, d=256, V=600, d_h=32, lengths=lens)
    b1 = np.random.default_rng(0).normal(size=32).astype(np.float32)
    b2 = np.array([0.75], dtype=np.float32)
    got = _run(gpu, w, b1=b1, b2=b2)
    off = oracle.offsets_from_lengths(lens)
    want = oracle.egtp(w.hidden, off, w.w_lm, oracle.Head(w.w1, w.w2, b1, b2))
    assert_egtp_close(got, want)
    hf = wl.bf16_bits_to_f32(w.hidden)
    for b, n in enumerate(lens):
        if n == 0:
            assert not got["pooled"][b].any() and got["lse"][b] == -np.inf
        if n == 1:
            assert np.array_equal(got["pooled"][b], hf[off[b]])     # weight is exactly 1


@pytest.mark.parametrize("alpha", [0.5, 4.0])
def test_temperature(gpu, alpha):
    w = _small_bf16(seed=13, B=4, d=128, V=700, d_h=16)
    got = _run(gpu, w, alpha=alpha)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2), alpha)
    assert_egtp_close(got, want)


def test_k_bin_head_expected_value(gpu):
    K = 20
    w = _small_bf16(seed=17, B=5, d=128, V=500, d_h=48)
    rng = np.random.default_rng(1)
    w2 = wl.to_bf16_bits(rng.normal(0, 1.0, size=(K, 48)).astype(np.float32))
    b2 = rng.normal(size=K).astype(np.float32)
    centers = np.linspace(16.0, 4096.0, K).astype(np.float32)
    got = _run(gpu, w, w2=w2, b2=b2, centers=centers)
    head = oracle.Head(w.w1, w2, None, b2, centers.astype(np.float64))
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, head)
    assert_egtp_close(got, want)


def test_positive_scalar_head_to_the_strict_relative_bar(gpu):
    # a scalar head with a large positive output bias: every prediction is far from zero, so the stated bar
    # (1e-2 relative) applies as it stands
    w = _small_bf16(seed=167, B=9, d=192, V=700, d_h=40)
    b2 = np.array([250.0], dtype=np.float32)
    b1 = (0.1 * np.random.default_rng(4).normal(size=40)).astype(np.float32)
    got = _run(gpu, w, b1=b1, b2=b2)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2, b1, b2))
    assert np.abs(want.pred).min() > 100.0
    assert_egtp_close(got, want)
    assert_pred_close(got["pred"], want.pred, strict=True)


def test_head_maximum_sizes(gpu):
    # widest head the interface takes: d_h = 16384 hidden units, K = 1024 bins, biases on both
    # layers; bf16 and fp32 weight storage
    K, d_h = 1024, 16384
    w = _small_bf16(seed=47, B=3, d=64, V=300, d_h=d_h, lengths=(9, 1, 40))
    rng = np.random.default_rng(2)
    w2f = (rng.normal(0, 1.0, size=(K, d_h)) / np.sqrt(d_h)).astype(np.float32)
    b1 = (0.05 * rng.normal(size=d_h)).astype(np.float32)
    b2 = rng.normal(size=K).astype(np.float32)
    centers = np.linspace(1.0, 8192.0, K).astype(np.float32)
    off = oracle.offsets_from_lengths(w.lengths)
    got = _run(gpu, w, w2=wl.to_bf16_bits(w2f), b1=b1, b2=b2, centers=centers)
    head = oracle.Head(w.w1, wl.to_bf16_bits(w2f), b1, b2, centers.astype(np.float64))
    want = oracle.egtp(w.hidden, off, w.w_lm, head)
    assert_egtp_close(got, want)
    assert want.pred.min() >= 1.0                       # expected values over positive centres: no floor needed
    assert_pred_close(got["pred"], want.pred, strict=True)
    # fp32 storage of the same head
    td = gpu.to_device
    w1f = wl.bf16_bits_to_f32(w.w1)
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w1f), td(w2f), td(b1), td(b2), td(centers)))
    out = _np(sc.score(td(w.hidden), _offsets_on_gpu(gpu, sc, w.lengths)))
    head = oracle.Head(w1f, w2f, b1, b2, centers.astype(np.float64))
    assert_egtp_close(out, oracle.egtp(w.hidden, off, w.w_lm, head))
    sc.close()


@pytest.mark.parametrize("storage", ["bf16", "f32"])
def test_k_bin_head_hands_out_its_distribution(gpu, storage):
    """Eq. 6: the scoring calls of a K-bin head also return p-hat, the softmax the predicted length is the
    expectation of -- element by element against the oracle, rows summing to 1, for EGTP and for a PLP step."""
    import torch
    K, d_h, d = 20, 48, 64
    w = _small_bf16(seed=149, B=5, d=d, V=300, d_h=d_h, lengths=(9, 1, 40, 0, 17))
    rng = np.random.default_rng(3)
    w2f = (rng.normal(0, 2.0, size=(K, d_h)) / np.sqrt(d_h)).astype(np.float32)
    b1 = (0.05 * rng.normal(size=d_h)).astype(np.float32)
    b2 = rng.normal(size=K).astype(np.float32)
    centers = np.linspace(16.0, 4096.0, K).astype(np.float32)
    td = gpu.to_device
    if storage == "bf16":
        w1s, w2s = w.w1, wl.to_bf16_bits(w2f)
    else:
        w1s, w2s = wl.bf16_bits_to_f32(w.w1), w2f
    head_dev = gpu.make_head(td(w1s), td(w2s), td(b1), td(b2), td(centers))
    sc = gpu.Scorer(td(w.w_lm), head_dev)
    off = _offsets_on_gpu(gpu, sc, w.lengths)
    B, T = w.spec.B, w.T
    out = dict(entropy=torch.empty(T, device="cuda"), pooled=torch.empty(B, d, device="cuda"),
               lse=torch.empty(B, device="cuda"), pred=torch.empty(B, device="cuda"))
    p_hat = torch.full((B, K), float("nan"), device="cuda")
    gpu.egtp_score_dist(sc.ctx, td(w.hidden), off, None, B, T, sc.workspace(T, B), out["entropy"], out["pooled"],
                        out["lse"], out["pred"], p_hat)
    head = oracle.Head(w1s, w2s, b1, b2, centers.astype(np.float64))
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, head)
    want_p, want_y = oracle.bin_decode(oracle.head_raw(want.pooled, head), centers)
    got_p = p_hat.cpu().numpy().astype(np.float64)
    assert np.abs(got_p - want_p).max() <= 2e-4 and np.abs(got_p.sum(axis=1) - 1.0).max() <= 1e-5
    assert_egtp_close(_np(out), want)
    assert np.abs(got_p @ centers.astype(np.float64) - out["pred"].cpu().numpy()).max() <= 1e-3 * centers.max()
    # one PLP step: the remaining-length head (the same one here) and its distribution
    g = wl.decode_hidden(w.spec, 1)
    pooled, lse = out["pooled"].clone(), out["lse"].clone()
    rem, p_rem = torch.empty(B, device="cuda"), torch.full((B, K), float("nan"), device="cuda")
    gpu.plp_step_dist(sc.ctx, td(g), None, None, None, B, B, pooled, lse, sc.workspace(B, B), None, rem, p_rem)
    r = oracle.plp(w.hidden, oracle.offsets_from_lengths(w.lengths), [g], w.w_lm, head)[0]
    rp, _ = oracle.bin_decode(oracle.head_raw(r.pooled, head), centers)
    assert np.abs(p_rem.cpu().numpy() - rp).max() <= 2e-4
    assert_pred_close(rem.cpu().numpy(), r.pred)
    sc.close()
    # a scalar head has no distribution: refused before anything is launched
    sc1 = _scorer(gpu, w)
    with pytest.raises(gpu.EgtpError) as e:
        gpu.egtp_score_dist(sc1.ctx, td(w.hidden), off, None, B, T, sc1.workspace(T, B), out["entropy"], out["pooled"],
                            out["lse"], out["pred"], p_hat)
    assert e.value.status == 2
    sc1.close()


def test_two_heads_of_unequal_width_share_the_workspace(gpu):
    """fp32 storage, head_len wider than head_rem (4096 against 4032 rows: the narrower head is cut into more
    slices along d and needs MORE partial planes).  The workspace is exactly egtp_workspace_bytes with a guard
    band behind it that no call may touch; both heads against the oracle."""
    import torch
    d, V, B = 320, 300, 3                      # d / 16 = 20 slices possible: 17 (4032 rows) against 16 (4096 rows)
    spec = wl.scaled(wl.SPECS["tiny"], seed=151, B=B, d=d, V=V, d_h=4096, lengths=(5, 1, 9))
    w = wl.make(spec)
    rng = np.random.default_rng(5)
    rem_w1 = rng.normal(0, d ** -0.5, size=(4032, d)).astype(np.float32)
    rem_w2 = rng.normal(0, 4032 ** -0.5, size=(1, 4032)).astype(np.float32)
    td = gpu.to_device
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w.w1), td(w.w2)), gpu.make_head(td(rem_w1), td(rem_w2)))
    need = gpu.egtp_workspace_bytes(sc.ctx, w.T, B)
    GUARD = 1 << 20
    buf = torch.full((need + GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    off = _offsets_on_gpu(gpu, sc, w.lengths)
    out = dict(entropy=torch.empty(w.T, device="cuda"), pooled=torch.empty(B, d, device="cuda"),
               lse=torch.empty(B, device="cuda"), pred=torch.empty(B, device="cuda"))
    gpu.egtp_score(sc.ctx, td(w.hidden), off, None, B, w.T, buf[:need], out["entropy"], out["pooled"], out["lse"],
                   out["pred"])
    g = wl.decode_hidden(spec, 1)
    pooled, lse, rem = out["pooled"].clone(), out["lse"].clone(), torch.empty(B, device="cuda")
    gpu.plp_step(sc.ctx, td(g), None, None, None, B, B, pooled, lse, buf[:need], None, rem)
    torch.cuda.synchronize()
    assert bool((buf[need:] == 0x5A).all()), "a call wrote behind its workspace"
    ooff = oracle.offsets_from_lengths(w.lengths)
    assert_egtp_close(_np(out), oracle.egtp(w.hidden, ooff, w.w_lm, oracle.Head(w.w1, w.w2)))
    r = oracle.plp(w.hidden, ooff, [g], w.w_lm, oracle.Head(rem_w1, rem_w2))[0]
    assert_pred_close(rem.cpu().numpy(), r.pred)
    sc.close()


def test_context_on_a_packed_lm_head_alone(gpu):
    """A bf16 context needs no row-major W_lm once a packed copy exists: pack with one context, free the
    original, adopt the packed copy in a context created with w_lm = NULL -- same bits out."""
    import torch
    w = _small_bf16(seed=157, B=3, d=96, V=700, d_h=16, lengths=(30, 300, 2))
    td = gpu.to_device
    w_lm_dev = td(w.w_lm)
    a = gpu.Scorer(w_lm_dev, gpu.make_head(td(w.w1), td(w.w2)))
    off = _offsets_on_gpu(gpu, a, w.lengths)
    ref = _np(a.score(td(w.hidden), off))
    packed = a._w_packed
    cfg = gpu.egtp_config()
    cfg.vocab, cfg.d, cfg.dtype, cfg.w_lm, cfg.alpha = w.spec.V, w.spec.d, gpu.EGTP_BF16, None, 1.0
    head_mem = (td(w.w1), td(w.w2))                               # the struct only borrows device memory
    cfg.head_len = gpu.make_head(*head_mem)
    ctx = gpu.egtp_create(cfg)
    B, T, d = w.spec.B, w.T, w.spec.d
    out = [torch.empty(T, device="cuda"), torch.empty(B, d, device="cuda"), torch.empty(B, device="cuda"),
           torch.empty(B, device="cuda")]
    ws = torch.empty(gpu.egtp_workspace_bytes(ctx, T, B), dtype=torch.uint8, device="cuda")
    with pytest.raises(gpu.EgtpError) as e:                       # nothing to read the LM head from yet
        gpu.egtp_score(ctx, td(w.hidden), off, None, B, T, ws, *out)
    assert e.value.status == 1
    with pytest.raises(gpu.EgtpError) as e:                       # and nothing to pack from
        gpu.egtp_pack_w_lm(ctx, torch.empty_like(packed))
    assert e.value.status == 1
    gpu.egtp_adopt_packed_w_lm(ctx, packed)
    del w_lm_dev
    ws = torch.empty(gpu.egtp_workspace_bytes(ctx, T, B), dtype=torch.uint8, device="cuda")
    gpu.egtp_score(ctx, td(w.hidden), off, None, B, T, ws, *out)
    for k, t in zip(("entropy", "pooled", "lse", "pred"), out):
        assert np.array_equal(t.cpu().numpy(), ref[k]), k
    gpu.egtp_destroy(ctx)
    a.close()


def test_malformed_device_offsets_stay_inside_the_buffers(gpu):
    """Device-side offsets are the caller's word (no host mirror given): whatever they hold, the pooling kernels
    clamp every token index to [0, T] -- the numbers are then meaningless, the accesses are not wild."""
    import torch
    w = _small_bf16(seed=163, B=4, d=64, V=300, d_h=8, lengths=(40, 200, 3, 57))
    sc = _scorer(gpu, w)
    hd = gpu.to_device(w.hidden)
    T, B = w.T, 4
    for bad in ([0, 40, 240, 243, T + 5000], [0, 500, 100, 243, T], [0, -7, 240, 243, T]):
        off = torch.tensor(bad, dtype=torch.int32).cuda()
        out = sc.score(hd, off)
        pooled, _ = sc.pool_ablation(hd, off, gpu.EGTP_POOL_AVERAGE)
        last, _ = sc.pool_ablation(hd, off, gpu.EGTP_POOL_LAST)
        torch.cuda.synchronize()
        assert out["pooled"].shape == (B, 64) and pooled.shape == (B, 64) and last.shape == (B, 64)
    good = _np(sc.score(hd, _offsets_on_gpu(gpu, sc, w.lengths)))        # the context is still fine afterwards
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(good, want)
    sc.close()


@pytest.mark.parametrize("B", [1, 63, 64, 65, 130])
def test_head_batch_tile_boundaries(gpu, B):
    # the first head layer works on 64-sequence tiles and slices d into more pieces the fewer tiles
    # there are: batches around the tile boundaries, one token per sequence so that pooled = token
    w = _small_bf16(seed=53 + B, B=B, d=320, V=257, d_h=72, lengths=tuple([1] * B))
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, np.arange(B + 1, dtype=np.int32), w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


def test_many_token_blocks_few_vocabulary_tiles(gpu):
    # 11 token blocks (one ragged group of 8 + 3) against 3 vocabulary tiles: the unit remap has to
    # cope with a last group that is not full and with fewer vocabulary ranges than asked for
    w = _small_bf16(seed=59, B=4, d=64, V=600, d_h=8, lengths=(700, 1100, 1, 900))
    assert (w.T + 255) // 256 == 11
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


@pytest.mark.parametrize("d,B,len_mu,n_points", [(96, 24, 6.7, 1), (32, 40, 6.72, 2)])
def test_paced_multi_tile_sweep_every_token(gpu, d, B, len_mu, n_points):
    """The launch configuration the serving benchmark runs -- several vocabulary tiles per workgroup (running
    maximum rescaled from tile to tile, the first half step of a tile issued behind the fold of the previous
    one) with the cohort pacing switched on -- at a shape the oracle sweeps in full: a small hidden size
    against many tokens and a large vocabulary.  Every token's entropy, every pooled vector and prediction."""
    V = 128037                                         # 501 tiles, the last one ragged
    w = wl.make(wl.scaled(wl.SPECS["mid"], seed=77 + d, B=B, d=d, V=V, d_h=48, len_mu=len_mu, len_sigma=0.7,
                          len_lo=16, len_hi=4000))
    plan = gpu.egtp_launch_plan_query(gpu.EGTP_BF16, d, V, w.T)
    assert plan.paced == 1 and plan.tiles_per_range > 4 * n_points, (w.T, plan.tiles_per_range)
    assert plan.vocab_tiles % plan.tiles_per_range != 0          # the last range is shorter and leaves early
    assert w.T % 256 != 0 and plan.token_blocks % 8 != 0           # ragged last block, ragged last group of blocks
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


def test_large_hidden_size(gpu):
    # d = 16384: 512 K steps per vocabulary tile through the ring; small T and V keep the oracle quick
    w = _small_bf16(seed=61, B=2, d=16384, V=300, d_h=8, lengths=(3, 70))
    got = _run(gpu, w)
    want = oracle.egtp(w.hidden, [0, 3, 73], w.w_lm, oracle.Head(w.w1, w.w2))
    assert_egtp_close(got, want)


def test_deterministic_and_batch_invariant(gpu):
    w = _small_bf16(seed=19, B=5, d=256, V=1500, d_h=32)
    sc = _scorer(gpu, w)
    off = _offsets_on_gpu(gpu, sc, w.lengths)
    hd = gpu.to_device(w.hidden)
    a = _np(sc.score(hd, off))
    b = _np(sc.score(hd, off))
    for k in a:
        assert np.array_equal(a[k], b[k]), k                       # run-to-run bit identical
    offs = oracle.offsets_from_lengths(w.lengths)
    for s in (0, 3):                                               # a sequence scored alone
        import torch
        one = _np(sc.score(hd[offs[s]:offs[s + 1]].contiguous(), torch.tensor([0, w.lengths[s]], dtype=torch.int32).cuda()))
        assert np.abs(one["entropy"] - a["entropy"][offs[s]:offs[s + 1]]).max() < 1e-5
        assert rel_l2(one["pooled"][0], a["pooled"][s]) < 1e-5


def test_two_contexts_overlap_on_two_streams(gpu):
    """Two contexts, each with its own workspace, scoring on two streams at once (a serving engine with more
    than one stream): every overlapped call gives, bit for bit, what the same call gives alone.  One of the two
    shapes runs with the cohort pacing on, whose counters live in the workspace and whose waits are bounded, so
    workgroups of the other launch sitting between a cohort's members may slow it down but change nothing."""
    import torch
    wa = _small_bf16(seed=201, B=9, d=32, V=128037, d_h=24, lengths=(400, 731, 290, 1, 512, 640, 77, 333, 516))
    plan = gpu.egtp_launch_plan_query(gpu.EGTP_BF16, 32, 128037, wa.T)
    assert plan.paced == 1 and plan.tiles_per_range >= 24          # one round of workgroups, six pacing points
    wb = _small_bf16(seed=202, B=7, d=512, V=5000, d_h=64, lo=30, hi=500)
    jobs = []
    for w in (wa, wb):
        sc = _scorer(gpu, w)
        off = _offsets_on_gpu(gpu, sc, w.lengths)
        hd = gpu.to_device(w.hidden)
        sc.workspace(w.T, len(w.lengths))                            # allocated before any stream forks
        alone = _np(sc.score(hd, off))
        assert_egtp_close(alone, oracle.egtp(w.hidden, oracle.offsets_from_lengths(w.lengths), w.w_lm,
                                             oracle.Head(w.w1, w.w2)))
        outs = [dict(entropy=torch.empty(w.T, dtype=torch.float32, device="cuda"),
                     pooled=torch.empty(len(w.lengths), w.spec.d, dtype=torch.float32, device="cuda"),
                     lse=torch.empty(len(w.lengths), dtype=torch.float32, device="cuda"),
                     pred=torch.empty(len(w.lengths), dtype=torch.float32, device="cuda")) for _ in range(2)]
        jobs.append((sc, hd, off, alone, outs, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(3):
        for sc, hd, off, _, outs, st in jobs:
            with torch.cuda.stream(st):
                for o in outs:                                       # two calls back to back on each stream
                    sc.score(hd, off, out=o)
        torch.cuda.synchronize()
        for _, _, _, alone, outs, _ in jobs:
            for o in outs:
                got = _np(o)
                for k in alone:
                    assert np.array_equal(got[k], alone[k]), (rep, k)
                o["entropy"].fill_(float("nan"))
                o["pooled"].fill_(float("nan"))
        torch.cuda.synchronize()


def test_vocabulary_permutation_invariance(gpu):
    w = _small_bf16(seed=23, B=2, d=128, V=1300, d_h=8)
    a = _run(gpu, w)
    perm = np.random.default_rng(0).permutation(1300)
    w.w_lm = np.ascontiguousarray(w.w_lm[perm])
    b = _run(gpu, w)
    assert np.abs(a["entropy"] - b["entropy"]).max() < 2e-5


def test_token_order_invariance_inside_a_sequence(gpu):
    """Eq. 2-4 do not look at positions: permuting the tokens of each sequence permutes the entropies and
    leaves pooled vector, lse and prediction unchanged (up to the order of the fp32 sums)."""
    lens = (300, 1, 77, 130)
    w = _small_bf16(seed=47, B=4, d=128, V=700, d_h=16, lengths=lens)
    a = _run(gpu, w)
    off = oracle.offsets_from_lengths(lens)
    rng = np.random.default_rng(1)
    perm = np.concatenate([off[b] + rng.permutation(lens[b]) for b in range(len(lens))])
    w.hidden = np.ascontiguousarray(w.hidden[perm])
    b = _run(gpu, w)
    assert np.array_equal(a["entropy"][perm], b["entropy"])          # a token's entropy depends on nothing else
    for s in range(len(lens)):
        assert rel_l2(b["pooled"][s], a["pooled"][s]) < 1e-5
    assert np.abs(a["lse"] - b["lse"]).max() < 1e-5
    assert_pred_close(b["pred"], a["pred"].astype(np.float64))


def test_ablation_poolers(gpu):
    lens = (4, 0, 33, 1)
    w = _small_bf16(seed=29, B=4, d=128, V=300, d_h=16, lengths=lens)
    sc = _scorer(gpu, w)
    off = _offsets_on_gpu(gpu, sc, lens)
    ooff = oracle.offsets_from_lengths(lens)
    head = oracle.Head(w.w1, w.w2)
    for kind in (gpu.EGTP_POOL_AVERAGE, gpu.EGTP_POOL_MAX, gpu.EGTP_POOL_LAST):
        pooled, pred = sc.pool_ablation(gpu.to_device(w.hidden), off, kind)
        want = oracle.pool_ablation(w.hidden, ooff, kind)
        got = pooled.cpu().numpy()
        assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
        assert_pred_close(pred.cpu().numpy(), oracle.predict(want, head))
    # fp32 storage too
    wt = wl.make(wl.SPECS["tiny"])
    sc = _scorer(gpu, wt)
    off = _offsets_on_gpu(gpu, sc, wt.lengths)
    pooled, _ = sc.pool_ablation(gpu.to_device(wt.hidden), off, gpu.EGTP_POOL_AVERAGE)
    want = oracle.pool_ablation(wt.hidden, oracle.offsets_from_lengths(wt.lengths), oracle.POOL_AVERAGE)
    assert np.abs(pooled.cpu().numpy() - want).max() < 1e-5


def test_pooling_unit_boundaries(gpu):
    """Sequences just below, at and above one and two pooling units (128 tokens per workgroup), an empty
    one and a long one: weighted pooling (Eq. 3-4) and the three ablation poolers against the oracle."""
    lens = (127, 128, 129, 0, 255, 256, 257, 1, 700)
    w = _small_bf16(seed=41, B=len(lens), d=136, V=300, d_h=16, lengths=lens)
    got = _run(gpu, w)
    ooff = oracle.offsets_from_lengths(lens)
    head = oracle.Head(w.w1, w.w2)
    assert_egtp_close(got, oracle.egtp(w.hidden, ooff, w.w_lm, head))
    sc = _scorer(gpu, w)
    off = _offsets_on_gpu(gpu, sc, lens)
    for kind in (gpu.EGTP_POOL_AVERAGE, gpu.EGTP_POOL_MAX, gpu.EGTP_POOL_LAST):
        pooled, _ = sc.pool_ablation(gpu.to_device(w.hidden), off, kind, want_pred=False)
        want = oracle.pool_ablation(w.hidden, ooff, kind)
        assert np.abs(pooled.cpu().numpy() - want).max() <= 1e-5 * max(1.0, np.abs(want).max()), kind


# ----------------------------------------------------------------------------- PLP (Eq. 8)
def _plp_setup(gpu, seed=31, B=5, d=256, V=900, d_h=24, steps=4):
    w = _small_bf16(seed=seed, B=B, d=d, V=V, d_h=d_h, lo=1, hi=60)
    rng = np.random.default_rng(seed + 1)
    rem_w1 = wl.to_bf16_bits(rng.normal(0, d ** -0.5, size=(d_h, d)).astype(np.float32))
    rem_w2 = wl.to_bf16_bits(rng.normal(0, d_h ** -0.5, size=(1, d_h)).astype(np.float32))
    gen = [wl.decode_hidden(w.spec, t + 1) for t in range(steps)]
    td = gpu.to_device
    sc = _scorer(gpu, w, head_rem=gpu.make_head(td(rem_w1), td(rem_w2)))
    return w, sc, gen, oracle.Head(rem_w1, rem_w2)


def test_plp_steps_match_egtp_on_concatenation(gpu):
    import torch
    w, sc, gen, head_rem = _plp_setup(gpu)
    off = _offsets_on_gpu(gpu, sc, w.lengths)
    out = sc.score(gpu.to_device(w.hidden), off)
    pooled, lse = out["pooled"].clone(), out["lse"].clone()
    want = oracle.plp(w.hidden, oracle.offsets_from_lengths(w.lengths), gen, w.w_lm, head_rem)
    for t, g in enumerate(gen):
        ent = torch.empty(w.spec.B, dtype=torch.float32, device="cuda")
        pred = sc.step(gpu.to_device(g), pooled, lse, entropy_out=ent)
        r = want[t]
        new_tok = oracle.offsets_from_lengths(np.asarray(w.lengths) + t + 1)[1:] - 1   # last token of each sequence
        assert np.abs(ent.cpu().numpy() - r.entropy[new_tok]).max() <= TOL_ENTROPY_ABS
        for b in range(w.spec.B):
            assert rel_l2(pooled[b].cpu().numpy(), r.pooled[b]) <= TOL_POOLED_REL_L2
        assert np.abs(lse.cpu().numpy() - r.lse).max() <= TOL_LSE_ABS
        assert_pred_close(pred.cpu().numpy(), r.pred)


def test_plp_from_empty_state_with_slots_and_checkpoint(gpu):
    import torch
    w, sc, gen, head_rem = _plp_setup(gpu, seed=37, steps=6)
    B, d = w.spec.B, w.spec.d
    S = B + 3
    slot = np.array([6, 0, 3, 7, 2], dtype=np.int32)
    slot_dev = torch.from_numpy(slot).cuda()
    pooled = torch.zeros(S, d, dtype=torch.float32, device="cuda")
    lse = torch.full((S,), -math.inf, dtype=torch.float32, device="cuda")
    empty = np.zeros((0, d), dtype=np.uint16)
    want = oracle.plp(empty, np.zeros(B + 1, np.int32), gen, w.w_lm, head_rem)
    snap = None
    for t, g in enumerate(gen):
        pred = sc.step(gpu.to_device(g), pooled, lse, slot_dev=slot_dev)
        if t == 2:
            snap = (pooled.clone(), lse.clone())
        for b in range(B):
            assert rel_l2(pooled[slot[b]].cpu().numpy(), want[t].pooled[b]) <= TOL_POOLED_REL_L2
        assert_pred_close(pred.cpu().numpy(), want[t].pred)
    unused = [s for s in range(S) if s not in slot]
    assert not pooled[unused].any().item() and torch.isinf(lse[unused]).all().item()
    # resume from the snapshot: bit-identical continuation
    p2, l2 = snap
    for g in gen[3:]:
        sc.step(gpu.to_device(g), p2, l2, slot_dev=slot_dev)
    assert torch.equal(p2, pooled) and torch.equal(l2, lse)


def test_plp_ragged_chunk_fold_equals_single_folds(gpu):
    import torch
    w, sc, gen, head_rem = _plp_setup(gpu, seed=41, steps=5)
    B = w.spec.B
    off = _offsets_on_gpu(gpu, sc, w.lengths)
    out = sc.score(gpu.to_device(w.hidden), off)
    # ragged fold: sequence b receives chunk_len[b] of the generated tokens in one call
    chunk_len = np.array([5, 0, 3, 1, 5], dtype=np.int32)
    rows = [gen[s][b] for b in range(B) for s in range(chunk_len[b])]
    chunk = np.stack(rows)
    coff = oracle.offsets_from_lengths(chunk_len)
    pooled, lse = out["pooled"].clone(), out["lse"].clone()
    pred = sc.step(gpu.to_device(chunk), pooled, lse, offsets_new_dev=torch.from_numpy(coff).cuda(),
                   offsets_new_host=coff)
    # oracle: EGTP over prompt + that sequence's chunk
    poff = oracle.offsets_from_lengths(w.lengths)
    cat, lens = [], []
    for b in range(B):
        cat.append(w.hidden[poff[b]:poff[b + 1]])
        cat.append(chunk[coff[b]:coff[b + 1]])
        lens.append(int(w.lengths[b] + chunk_len[b]))
    want = oracle.egtp(np.concatenate(cat), oracle.offsets_from_lengths(lens), w.w_lm, head_rem)
    for b in range(B):
        assert rel_l2(pooled[b].cpu().numpy(), want.pooled[b]) <= TOL_POOLED_REL_L2
    assert np.abs(lse.cpu().numpy() - want.lse).max() <= TOL_LSE_ABS
    assert_pred_close(pred.cpu().numpy(), want.pred)


# ----------------------------------------------------------------------------- error paths (host side)
def test_error_codes_before_any_launch(gpu):
    import torch
    w = _small_bf16(seed=43, B=2, d=64, V=300, d_h=8, lengths=(3, 4))
    sc = _scorer(gpu, w)
    hd = gpu.to_device(w.hidden)
    off = torch.tensor([0, 3, 7], dtype=torch.int32).cuda()
    outs = [torch.empty(7, device="cuda"), torch.empty(2, 64, device="cuda"), torch.empty(2, device="cuda"),
            torch.empty(2, device="cuda")]
    ws = sc.workspace(7, 2)

    def status(fn):
        with pytest.raises(gpu.EgtpError) as e:
            fn()
        return e.value.status

    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, [0, 4, 3], 2, 7, ws, *outs)) == 3      # decreasing
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, [1, 3, 7], 2, 7, ws, *outs)) == 3      # offsets[0] != 0
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, [0, 3, 6], 2, 7, ws, *outs)) == 3      # offsets[B] != T
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, None, 2, 7, ws[:256], *outs)) == 5     # too small
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, None, 2, 7, ws[16:], *outs)) == 5      # misaligned
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, off, None, -1, 7, ws, *outs)) == 2
    assert status(lambda: gpu.egtp_score(sc.ctx, hd, None, None, 2, 7, ws, *outs)) == 1
    assert status(lambda: gpu.plp_step(sc.ctx, hd, None, None, None, 2, 7, outs[1], outs[2], ws, None, outs[3])) == 2
    gpu.egtp_score(sc.ctx, hd, off, [0, 3, 7], 0, 0, None, None, None, None, None)               # B == 0: nothing to do
    gpu.egtp_score(sc.ctx, hd, off, [0, 3, 7], 2, 7, ws, *outs)                                  # and the good call works
    torch.cuda.synchronize()


def test_mfma_probe_runs_and_checks_arguments(gpu):
    """The measurement aid: rates are positive and below the chip's clock-limited ceiling; bad arguments
    are turned into status codes before anything is launched."""
    import torch
    sc = _scorer(gpu, wl.make(wl.SPECS["tiny"]))
    n = gpu.egtp_mfma_probe_sink_floats()
    assert n == 1024 * 256
    sink = torch.empty(n, dtype=torch.float32, device="cuda")
    for random_operands in (False, True):
        r = gpu.egtp_mfma_probe(sc.ctx, sink, 2000, random_operands, 2)
        assert r.shape == (2,) and (r > 50.0).all() and (r < 2600.0).all(), r
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())
    assert float(gpu.egtp_mfma_probe(sc.ctx, sink, 1, False, 1)[0]) >= 0.0
    for bad in (dict(iters=0), dict(launches=0), dict(launches=65)):
        kw = dict(iters=10, launches=1)
        kw.update(bad)
        with pytest.raises(gpu.EgtpError):
            gpu.egtp_mfma_probe(sc.ctx, sink, kw["iters"], False, kw["launches"])
    with pytest.raises(gpu.EgtpError):
        gpu.egtp_mfma_probe(sc.ctx, sink[:1000], 10, False, 1)


def test_hbm_read_probe_reads_every_word_once(gpu):
    """The streaming-read measurement: the per-thread XOR words it leaves in its sink fold to the XOR of the
    whole buffer (a piece read twice or skipped would break that, ragged 16-byte tail included), rates are
    positive and finite, and bad arguments become status codes before any launch."""
    import torch
    sc = _scorer(gpu, wl.make(wl.SPECS["tiny"]))
    nsink = gpu.egtp_hbm_read_probe_sink_bytes()
    assert nsink == 8192 * 256 * 4
    sink = torch.empty(nsink, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(11)
    for nbytes in ((1 << 20), (1 << 20) + 16 * 12345, (64 << 20) + 16 * 7 + 8):
        buf = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
        r = gpu.egtp_hbm_read_probe(sc.ctx, buf, sink, 2)
        assert r.shape == (2,) and (r > 0.0).all() and (r < 2.0e4).all(), r   # cache-resident sizes
        torch.cuda.synchronize()
        words = buf[:nbytes // 16 * 16].view(torch.int32).cpu().numpy()
        want = int(np.bitwise_xor.reduce(words))
        got = int(np.bitwise_xor.reduce(sink.view(torch.int32).cpu().numpy()))
        assert got == want, nbytes
    buf = torch.zeros(2 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(gpu.EgtpError):
        gpu.egtp_hbm_read_probe(sc.ctx, buf[:1000], sink, 1)          # under 1 MiB
    with pytest.raises(gpu.EgtpError):
        gpu.egtp_hbm_read_probe(sc.ctx, buf[8:], sink, 1)             # not 16-byte aligned
    with pytest.raises(gpu.EgtpError):
        gpu.egtp_hbm_read_probe(sc.ctx, buf, sink[:nsink - 4], 1)     # sink too small
    for launches in (0, 65):
        with pytest.raises(gpu.EgtpError):
            gpu.egtp_hbm_read_probe(sc.ctx, buf, sink, launches)


def test_head_keeps_the_pooled_vector_in_fp32(gpu):
    """The head must not re-round its fp32 input to bf16 on its way to the matrix cores: against the
    oracle's head evaluated in fp64 on the GPU's own pooled vectors, predictions agree to fp32
    accumulation noise, and the same head on inputs cut to one bf16 piece misses that bar."""
    w = wl.make(wl.SPECS["mid"])
    got = _run(gpu, w)
    pooled = got["pooled"].astype(np.float64)
    head = oracle.Head(w.w1, w.w2)
    want = oracle.predict(pooled, head)
    # scale of the sum each prediction is: sum_j |w2_j| * sum_k |W1_jk x_k|
    w1 = wl.bf16_bits_to_f32(w.w1).astype(np.float64)
    w2 = wl.bf16_bits_to_f32(w.w2).astype(np.float64)
    scale = (np.abs(pooled) @ np.abs(w1).T) @ np.abs(w2).reshape(-1)
    err = np.abs(got["pred"].astype(np.float64) - want) / scale
    bar = 1e-6
    assert err.max() < bar, err.max()
    hi = (got["pooled"].view(np.uint32) & np.uint32(0xffff0000)).view(np.float32).astype(np.float64)
    assert (np.abs(oracle.predict(hi, head) - want) / scale).max() > 2 * bar


def test_plp_steps_replayed_from_a_graph(gpu):
    """The scoring calls only enqueue kernels on the caller's stream, so a decode loop can be captured in a
    HIP graph.  Three steps are captured once and replayed four times, with eager work and
    synchronisations in between; every replay must leave exactly what the same twelve eager steps leave."""
    import torch
    w, sc, gen, _ = _plp_setup(gpu, seed=43, steps=3)
    B, d = w.spec.B, w.spec.d
    hs = [gpu.to_device(g) for g in gen]

    def fresh():
        return (torch.zeros(B, d, dtype=torch.float32, device="cuda"),
                torch.full((B,), -math.inf, dtype=torch.float32, device="cuda"),
                [torch.empty(B, dtype=torch.float32, device="cuda") for _ in hs])

    ws = sc.workspace(B, B)
    pooled_e, lse_e, pred_e = fresh()
    pooled_g, lse_g, pred_g = fresh()
    # the first call on a device raises kernel attributes: keep that outside the capture
    warm_p, warm_l, warm_r = fresh()
    gpu.plp_step(sc.ctx, hs[0], None, None, None, B, B, warm_p, warm_l, ws, None, warm_r[0])
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for h, r in zip(hs, pred_g):
                gpu.plp_step(sc.ctx, h, None, None, None, B, B, pooled_g, lse_g, ws, None, r)
    torch.cuda.synchronize()
    ws_e = sc.workspace(B, B).clone()
    for replay in range(4):
        graph.replay()
        for h, r in zip(hs, pred_e):
            gpu.plp_step(sc.ctx, h, None, None, None, B, B, pooled_e, lse_e, ws_e, None, r)
        scratch = torch.randn(1 << 16, device="cuda").sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(pooled_g, pooled_e) and torch.equal(lse_g, lse_e), replay
        for a, b in zip(pred_g, pred_e):
            assert torch.equal(a, b), replay
        assert bool(torch.isfinite(scratch))


def test_paced_score_replayed_from_a_graph(gpu):
    """The prefill call with the cohort pacing on (its counters are cleared by a kernel, not by a memset
    node) captured in a HIP graph together with the offset scan: four replays, eager work and a poisoned
    workspace in between, each bit-identical to the eager call."""
    import torch
    w = _small_bf16(seed=211, B=9, d=32, V=128037, d_h=24, lengths=(400, 731, 290, 1, 512, 640, 77, 333, 516))
    assert gpu.egtp_launch_plan_query(gpu.EGTP_BF16, 32, 128037, w.T).paced == 1
    sc = _scorer(gpu, w)
    B, T, d = len(w.lengths), w.T, w.spec.d
    hd = gpu.to_device(w.hidden)
    lengths = torch.from_numpy(np.asarray(w.lengths, dtype=np.int32)).cuda()

    def outputs():
        return (torch.empty(B + 1, dtype=torch.int32, device="cuda"), torch.empty(T, dtype=torch.float32, device="cuda"),
                torch.empty(B, d, dtype=torch.float32, device="cuda"), torch.empty(B, dtype=torch.float32, device="cuda"),
                torch.empty(B, dtype=torch.float32, device="cuda"))

    ws = sc.workspace(T, B)
    eager = outputs()
    gpu.egtp_build_offsets(sc.ctx, lengths, B, eager[0], None, T)      # also the warm-up outside the capture
    gpu.egtp_score(sc.ctx, hd, eager[0], None, B, T, ws, *eager[1:])
    torch.cuda.synchronize()
    want = [t.clone() for t in eager]
    got = outputs()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            gpu.egtp_build_offsets(sc.ctx, lengths, B, got[0], None, T)
            gpu.egtp_score(sc.ctx, hd, got[0], None, B, T, ws, *got[1:])
    torch.cuda.synchronize()
    for replay in range(4):
        ws.fill_(0xff)                                                    # NaN patterns everywhere, counters included
        for t in got[1:]:
            t.fill_(float("nan"))
        graph.replay()
        scratch = torch.randn(1 << 16, device="cuda").sum()              # unrelated eager work between replays
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), replay
        assert bool(torch.isfinite(scratch))


@pytest.mark.parametrize("case", range(12))
def test_seeded_random_shapes_against_the_oracle(gpu, case):
    """Twelve seeded draws of batch size, ragged lengths (empty sequences included), hidden size,
    vocabulary, head width, biases, temperature and scalar or K-bin output, each against the oracle."""
    rng = np.random.default_rng(1000 + case)
    B = int(rng.integers(1, 10))
    lens = tuple(int(x) for x in np.where(rng.random(B) < 0.15, 0, rng.integers(1, 420, size=B)))
    d = 8 * int(rng.integers(1, 66))
    V = int(rng.integers(1, 3000))
    d_h = int(rng.integers(1, 70))
    alpha = float(rng.choice([0.5, 1.0, 1.0, 2.5]))
    w = _small_bf16(seed=2000 + case, B=B, d=d, V=V, d_h=d_h, lengths=lens)
    b1 = (0.1 * rng.normal(size=d_h)).astype(np.float32) if rng.random() < 0.5 else None
    if rng.random() < 0.5:
        K = int(rng.integers(2, 40))
        w2 = wl.to_bf16_bits(rng.normal(0, 1.0, size=(K, d_h)).astype(np.float32))
        b2 = rng.normal(size=K).astype(np.float32)
        centers = np.sort(rng.uniform(1.0, 4096.0, size=K)).astype(np.float32)
    else:
        w2, centers = w.w2, None
        b2 = rng.normal(size=1).astype(np.float32) if rng.random() < 0.5 else None
    got = _run(gpu, w, alpha=alpha, b1=b1, b2=b2, w2=w2, centers=centers)
    head = oracle.Head(w.w1, w2, b1, b2, None if centers is None else centers.astype(np.float64))
    want = oracle.egtp(w.hidden, oracle.offsets_from_lengths(lens), w.w_lm, head, alpha)
    assert_egtp_close(got, want)


@pytest.mark.parametrize("case", range(6))
def test_seeded_random_plp_histories_against_the_oracle(gpu, case):
    """Seeded decode histories: a random subset of the state slots is live at each call and receives a
    random number (0..70) of new tokens through `slot`; after every call each live slot must hold what
    the oracle computes from that slot's whole history (Eq. 8 as EGTP on the concatenation)."""
    import torch
    rng = np.random.default_rng(3000 + case)
    S = int(rng.integers(2, 8))                       # state slots
    d = 8 * int(rng.integers(2, 40))
    V = int(rng.integers(50, 2000))
    d_h = int(rng.integers(2, 40))
    w = _small_bf16(seed=4000 + case, B=S, d=d, V=V, d_h=d_h, lengths=tuple(int(x) for x in rng.integers(0, 90, size=S)))
    sc = _scorer(gpu, w)
    head = oracle.Head(w.w1, w.w2)
    poff = oracle.offsets_from_lengths(w.lengths)
    history = [w.hidden[poff[b]:poff[b + 1]] for b in range(S)]
    out = sc.score(gpu.to_device(w.hidden), _offsets_on_gpu(gpu, sc, w.lengths))
    pooled, lse = out["pooled"].clone(), out["lse"].clone()
    for call in range(4):
        live = np.sort(rng.choice(S, size=int(rng.integers(1, S + 1)), replace=False)).astype(np.int32)
        n_new = rng.integers(0, 71, size=live.size).astype(np.int32)
        if n_new.sum() == 0:
            n_new[0] = 1
        T_new = int(n_new.sum())
        chunk = wl.draw_hidden(w.spec, np.random.default_rng([3000 + case, call]), T_new)
        chunk = wl.to_bf16_bits(chunk) if chunk.dtype != np.uint16 else chunk
        coff = oracle.offsets_from_lengths(n_new)
        pred = sc.step(gpu.to_device(chunk), pooled, lse, offsets_new_dev=torch.from_numpy(coff).cuda(),
                       offsets_new_host=coff, slot_dev=torch.from_numpy(live).cuda())
        for i, sl in enumerate(live):
            history[sl] = np.concatenate([history[sl], chunk[coff[i]:coff[i + 1]]])
        lens = [history[sl].shape[0] for sl in live]
        want = oracle.egtp(np.concatenate([history[sl] for sl in live]), oracle.offsets_from_lengths(lens), w.w_lm, head)
        pooled_np, lse_np = pooled.cpu().numpy(), lse.cpu().numpy()
        for i, sl in enumerate(live):
            if lens[i] > 0:
                assert rel_l2(pooled_np[sl], want.pooled[i]) <= TOL_POOLED_REL_L2, (call, sl)
                assert abs(lse_np[sl] - want.lse[i]) <= TOL_LSE_ABS, (call, sl)
        assert_pred_close(pred.cpu().numpy(), want.pred)
