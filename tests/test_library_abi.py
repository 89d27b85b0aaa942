"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
public header declares, and rejects malformed configurations before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_11812_amd", "libegtp.so")
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))
                 if f.endswith(".h"))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2602_11812_amd.build import build_library
        build_library()
    return ctypes.CDLL(LIB)


def _declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(egtp_[a-z_]+|plp_step[a-z_]*)\s*\(", text)))


def test_header_declares_the_scoring_calls():
    names = _declared_functions()
    for must in ("egtp_create", "egtp_destroy", "egtp_workspace_bytes", "egtp_build_offsets", "egtp_score",
                 "plp_step", "egtp_pool_ablation", "egtp_status_string", "egtp_last_hip_error"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"


def test_binding_lists_the_same_symbols():
    from paper_2602_11812_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_status_strings(lib):
    lib.egtp_status_string.restype = ctypes.c_char_p
    seen = {lib.egtp_status_string(i) for i in range(10)}
    assert len(seen) == 10 and all(s for s in seen)


def test_create_rejects_bad_configs_without_a_device(lib):
    from paper_2602_11812_amd.binding import egtp_config
    lib.egtp_create.restype = ctypes.c_int
    ctx = ctypes.c_void_p()
    fake = 0x1000  # never dereferenced: validation happens first

    def cfg(**kw):
        c = egtp_config()
        c.d, c.vocab, c.dtype, c.w_lm, c.alpha = 256, 1000, 1, fake, 1.0
        c.head_len.d_h, c.head_len.n_out, c.head_len.wdtype = 32, 1, 1
        c.head_len.w1, c.head_len.w2 = fake, fake
        for k, v in kw.items():
            obj = c
            *path, leaf = k.split("__")
            for p in path:
                obj = getattr(obj, p)
            setattr(obj, leaf, v)
        return c

    def create(c):
        return lib.egtp_create(ctypes.byref(c), ctypes.byref(ctx))

    assert lib.egtp_create(None, ctypes.byref(ctx)) == 1
    assert create(cfg(dtype=7)) == 4
    assert create(cfg(d=0)) == 2
    assert create(cfg(d=100)) == 2                  # bf16 rows must be 16-byte aligned
    assert create(cfg(vocab=-5)) == 2
    assert create(cfg(w_lm=None, dtype=0, d=256)) in (0, 6)   # a context may live on a packed copy alone
    assert create(cfg(w_lm=None)) in (0, 6)
    assert create(cfg(dtype=0, d=699044)) == 2                # fp32: six bf16 segments must fit the kernel's reach
    assert create(cfg(dtype=0, d=699040)) in (0, 6)
    assert create(cfg(alpha=0.0)) == 8
    assert create(cfg(alpha=float("nan"))) == 8
    assert create(cfg(alpha=float("inf"))) == 8
    assert create(cfg(head_len__d_h=0)) == 2
    assert create(cfg(head_len__w1=None)) == 1
    assert create(cfg(head_len__wdtype=3)) == 4
    assert create(cfg(head_len__n_out=20)) == 1     # K-bin head without bin centres
    assert create(cfg(head_rem__w1=fake, head_rem__d_h=0)) == 2
    # a well-formed configuration gets as far as the device check
    st = create(cfg())
    assert st in (0, 6)
    if st == 0:
        lib.egtp_destroy.argtypes = [ctypes.c_void_p]
        lib.egtp_destroy(ctx)


def test_null_context_is_an_error_not_a_crash(lib):
    lib.egtp_workspace_bytes.restype = ctypes.c_size_t
    lib.egtp_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32]
    assert lib.egtp_workspace_bytes(None, 10, 1) == 0
    lib.egtp_score.restype = ctypes.c_int
    assert lib.egtp_score(None, None, None, None, 1, 1, None, 0, None, None, None, None, None) == 1
    lib.plp_step.restype = ctypes.c_int
    assert lib.plp_step(None, None, None, None, None, 1, 1, None, None, None, 0, None, None, None) == 1


def test_training_workspace_size_is_monotonic_and_rejects_bad_shapes(lib):
    f = lib.egtp_head_train_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int32] * 4
    prev = 0
    for B in (0, 1, 15, 16, 63, 64, 65, 128, 129, 1000, 4096):
        n = f(B, 4096, 1024, 20)
        assert n >= prev and n % 256 == 0
        # at least the activations, their gradients, dL/dz and the loss terms
        assert n >= 4 * (2 * B * 1024 + B * 20 + 2 * B)
        prev = n
    assert f(16, 4094, 1024, 20) == 0        # feature size must be a multiple of 4
    assert f(16, 4096, 0, 20) == 0 and f(16, 4096, 1024, 0) == 0 and f(-1, 4096, 1024, 20) == 0
    assert f(16, 4096, 16385, 20) == 0 and f(16, 4096, 1024, 1025) == 0


class _Plan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("tokens_per_block", "rows_per_tile", "token_blocks", "vocab_tiles",
                                               "vocab_ranges", "tiles_per_range", "paced")]


def test_launch_plan_query_needs_no_device_and_covers_the_vocabulary(lib):
    """The plan the fused kernel would be launched with: every vocabulary tile belongs to exactly one range,
    the token blocks cover the batch, and malformed shapes come back as status codes."""
    q = lib.egtp_launch_plan_query
    q.restype = ctypes.c_int
    q.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(_Plan)]
    for dtype in (0, 1):
        for d, V, T in ((4096, 151936, 137720), (4096, 151936, 512), (4096, 151936, 1), (64, 200, 10),
                        (4096, 128037, 24576), (8192, 32000, 100000), (256, 257, 0)):
            p = _Plan()
            assert q(dtype, d, V, T, ctypes.byref(p)) == 0
            assert p.tokens_per_block > 0 and p.rows_per_tile > 0
            assert p.vocab_tiles == -(-V // p.rows_per_tile)
            assert p.token_blocks == -(-T // p.tokens_per_block)
            assert 1 <= p.vocab_ranges <= p.vocab_tiles
            assert (p.vocab_ranges - 1) * p.tiles_per_range < p.vocab_tiles <= p.vocab_ranges * p.tiles_per_range
            assert p.paced in (0, 1) and not (p.paced and p.token_blocks < 8)
    p = _Plan()
    assert q(1, 4096, 151936, 137720, ctypes.byref(p)) == 0 and p.paced == 1     # the configuration that is timed
    assert q(1, 4096, 151936, 137720, None) == 1
    assert q(7, 4096, 151936, 10, ctypes.byref(p)) != 0
    for d, V, T in ((0, 10, 10), (10, 0, 10), (10, 10, -1), (10, 10, 1 << 31)):
        assert q(1, d, V, T, ctypes.byref(p)) != 0
