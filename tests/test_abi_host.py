"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
declared in include/fss.h, sizes its key buffers like the paper's closed form, and rejects
bad arguments before touching the device."""
import os
import re

import pytest

import paper_2006_04593_amd as fss
from paper_2006_04593_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fss.library_path()):
        fss.build()
    return fss.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fss.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fss_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_key_bytes(lib):
    assert fss.cmp_key_bytes(32, 64) == 808 * 64
    assert fss.eq_key_bytes(32, 64) == 544 * 64
    assert fss.cmp_key_bytes(32, 65) == 808 * 128          # padded to a wavefront
    assert fss.cmp_key_bytes(32, 1 << 22) == 808 << 22     # the paper's 808 bytes per element
    assert fss.cmp_key_bytes(8, 64) == 64 * (4 + 16 + 16 + 8 * 24 + 4)
    assert fss.eq_key_bytes(12, 64) == 64 * (4 + 16 + 8 + 12 * 16 + 4)
    for n in (0, -1, 33):
        assert fss.cmp_key_bytes(n, 64) == 0 and fss.eq_key_bytes(n, 64) == 0
    assert fss.cmp_key_bytes(32, 0) == 0
    assert fss.cmp_key_bytes(32, 1 << 40) == 808 << 40     # the largest batch a call takes
    assert fss.cmp_key_bytes(32, (1 << 40) + 1) == 0 and fss.eq_key_bytes(32, (1 << 64) - 1) == 0


def test_key_sizes_agree_with_the_oracle_layout(lib):
    import oracle
    for n in (1, 8, 12, 32):
        for batch in (1, 64, 1000):
            assert fss.cmp_key_bytes(n, batch) == oracle.key_bytes("cmp", n, batch)
            assert fss.eq_key_bytes(n, batch) == oracle.key_bytes("eq", n, batch)


def test_bad_arguments_are_rejected_on_the_host(lib):
    A = 0x10000                                       # any aligned non-null address; never dereferenced
    for f in (lib.fss_cmp_eval, lib.fss_eq_eval):
        assert f(2, 32, 8, A, A, A, None) == -1       # party
        assert f(-1, 32, 8, A, A, A, None) == -1
        assert f(0, 0, 8, A, A, A, None) == -1        # n
        assert f(0, 33, 8, A, A, A, None) == -1
        assert f(0, 32, 8, None, A, A, None) == -1    # NULL
        assert f(0, 32, 8, A, None, A, None) == -1
        assert f(0, 32, 8, A, A, None, None) == -1
        assert f(0, 32, 8, A + 16, A, A, None) == -1  # key buffer alignment
        assert f(0, 32, 8, A, A + 2, A, None) == -1
        assert f(0, 32, 0, None, None, None, None) == 0   # empty batch is a no-op
        assert f(0, 33, 0, None, None, None, None) == -1  # ... but n is still checked
    for f in (lib.fss_cmp_gen, lib.fss_eq_gen):
        B = A + (1 << 20)
        assert f(0, 8, A, A, A, A, A, B, None) == -1
        assert f(32, 8, None, A, A, A, A, B, None) == -1
        assert f(32, 8, A, A, A + 4, A, A, B, None) == -1     # seeds need 16-byte alignment
        assert f(32, 8, A, A, A, A, A, A, None) == -1         # overlapping key buffers
        assert f(32, 8, A, A, A, A, A, A + 256, None) == -1
        assert f(32, 0, None, None, None, None, None, None, None) == 0


def test_protocol_entry_points_reject_bad_arguments_on_the_host(lib):
    A = 0x10000
    assert lib.fss_sign_mask(0, 8, A, A, A, None) == -1
    assert lib.fss_sign_mask(32, 8, A + 8, A, A, None) == -1
    assert lib.fss_sign_mask(32, 0, None, None, None, None) == 0
    assert lib.fss_sign_eval(0, 32, 8, A, A, None, A, None) == -1            # second masked share missing
    assert lib.fss_relu_open(0, 32, 8, A, A, A, A, A, None, A, A, None) == -1
    assert lib.fss_relu_open(3, 32, 0, None, None, None, None, None, None, None, None, None) == -1
    assert lib.fss_relu_finish(0, 32, 8, A, A, A, A, A, A, A, None, None) == -1
    assert lib.fss_eq_mask(32, 8, A, None, A, None) == -1
    assert lib.fss_eq_masked_eval(0, 32, 8, A, A, A + 1, A, None) == -1
    assert lib.fss_argmax_diff_mask(32, 4, 1, A, A, A, None) == -1           # m < 2
    assert lib.fss_argmax_count_mask(2, 32, 4, 3, A, A, A, None) == -1
    assert lib.fss_maxpool_unroll(4, 2, 8, 3, 2, A, A, None) == -1            # window larger than the image
    assert lib.fss_maxpool_unroll(0, 8, 8, 2, 2, None, None, None) == 0
    assert lib.fss_mul_open(33, 8, A, A, A, A, A, A, None) == -1
    assert lib.fss_dot_finish(0, 32, 8, 0, A, A, A, A, A, A, A, A, None) == -1


def test_element_counts_that_would_overflow_are_rejected(lib):
    A, B = 0x10000, 0x10000 + (1 << 20)
    huge = (1 << 40) + 1
    assert lib.fss_cmp_eval(0, 32, huge, A, A, A, None) == -1
    assert lib.fss_eq_eval(0, 32, (1 << 64) - 1, A, A, A, None) == -1
    assert lib.fss_cmp_gen(32, huge, A, A, A, A, A, B, None) == -1
    assert lib.fss_sign_mask(32, huge, A, A, A, None) == -1
    assert lib.fss_relu_finish(0, 32, huge, A, A, A, A, A, A, A, A, None) == -1
    assert lib.fss_mul_open(32, huge, A, A, A, A, A, A, None) == -1
    assert lib.fss_argmax_diff_mask(32, 1 << 39, 3, A, A, A, None) == -1         # rows * m * (m - 1) > 2^40
    assert lib.fss_argmax_diff_mask(32, 1 << 62, 4, A, A, A, None) == -1         # would wrap around in 64 bits
    assert lib.fss_argmax_count_mask(0, 32, 1 << 39, 3, A, A, A, None) == -1
    assert lib.fss_dot_finish(0, 32, 1 << 39, 9, A, A, A, A, A, A, A, A, None) == -1
    assert lib.fss_maxpool_unroll(1 << 40, 4, 4, 2, 2, A, A, None) == -1
    assert lib.fss_cmp_chunked_key_bytes(32, huge, 256) == 0
    assert lib.fss_cmp_eval_streamed(0, 32, huge, 256, A, A, A, A, None, A) == -1


def test_streamed_evaluation_arguments(lib):
    A = 0x10000
    assert lib.fss_cmp_chunked_key_bytes(32, 1000, 256) == 808 * 1024          # 3 full chunks + 232 padded to 256
    assert lib.fss_cmp_chunked_key_bytes(32, 1024, 256) == 808 * 1024
    assert lib.fss_cmp_chunked_key_bytes(32, 1000, 100) == 0                   # chunk must be a multiple of 64
    assert lib.fss_cmp_chunked_key_bytes(0, 1000, 256) == 0
    S1, S2 = 0x1000, 0x2000                                                    # stand-ins; validation never dereferences
    assert lib.fss_cmp_eval_streamed(0, 32, 100, 100, A, A, A, A, S1, S2) == -1
    assert lib.fss_cmp_eval_streamed(0, 32, 100, 64, A, A, A, A, S1, S1) == -1    # one stream for both roles
    assert lib.fss_cmp_eval_streamed(0, 32, 100, 64, None, A, A, A, S1, S2) == -1
    assert lib.fss_cmp_eval_streamed(0, 32, 0, 64, None, None, None, None, S1, S2) == 0


def test_static_staging_arguments(lib):
    A, S1, S2 = 0x10000, 0x1000, 0x2000
    assert lib.fss_static_staging_bytes() == 32 << 20
    assert lib.fss_cmp_eval_streamed_static(0, 32, 100, 100, A, A, A, S1, S2) == -1       # chunk not a multiple of 64
    assert lib.fss_cmp_eval_streamed_static(0, 32, 100, 64, A, A, A, S1, S1) == -1        # one stream for both roles
    assert lib.fss_cmp_eval_streamed_static(2, 32, 100, 64, A, A, A, S1, S2) == -1
    assert lib.fss_cmp_eval_streamed_static(0, 32, 100, 20736 + 64, A, A, A, S1, S2) == -4   # beyond the built-in staging memory
    assert lib.fss_cmp_eval_streamed_static(0, 8, 100, 20736 + 64, None, A, A, S1, S2) == -1  # fits at n = 8; NULL keys
    assert lib.fss_cmp_eval_streamed_static(0, 32, 0, 64, None, None, None, S1, S2) == 0
    assert b"limit" in lib.fss_strerror(-4)


def test_clock_probe_arguments(lib):
    A = 0x10000
    assert lib.fss_clock_probe(None, 10, None) == -1
    assert lib.fss_clock_probe(A + 4, 10, None) == -1          # two u64: 8-byte alignment
    assert lib.fss_clock_probe(A, 0, None) == -1
    assert lib.fss_clock_probe(A, (1 << 20) + 1, None) == -1    # bounded: the probe always ends


def test_layout_switch_query(lib):
    # 512 elements per compute unit on a device; 0 where there is none to ask
    assert lib.fss_quad_layout_below() % 512 == 0


def test_strerror(lib):
    assert lib.fss_strerror(0) == b"success"
    for code in (-1, -2, -3, 17):
        assert len(lib.fss_strerror(code)) > 0


def test_binding_wants_gpu_tensors():
    torch = pytest.importorskip("torch")
    t = torch.zeros(8, dtype=torch.int32)
    with pytest.raises(ValueError, match="GPU tensor"):
        fss.cmp_eval(0, 32, 8, torch.zeros(fss.cmp_key_bytes(32, 8), dtype=torch.uint8), t, t, stream=0)


def test_binding_raises_with_the_code():
    with pytest.raises(fss.FssError) as e:
        fss.cmp_eval(5, 32, 4, None, None, None, stream=0)
    assert e.value.code == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_SO", str(tmp_path / "absent.so"))
    with pytest.raises(FileNotFoundError):
        fss.cmp_key_bytes(32, 64)
