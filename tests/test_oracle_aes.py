"""Pins for the oracle's AES-128 and PRG: FIPS-197 known answers, the OpenSSL tool, and
the Matyas-Meyer-Oseas definition G_m(s) = E_{k_m}(s) xor s (paper, section 3.1
"Implementation" and appendix C.1)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "aes128_known_answers.txt")


def known_answers():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, p, c = line.split()
                rows.append((bytes.fromhex(k), bytes.fromhex(p), bytes.fromhex(c)))
    return rows


def test_fips197_known_answers():
    rows = known_answers()
    assert len(rows) >= 2
    for key, pt, ct in rows:
        assert oracle.aes128_encrypt(key, pt) == ct


def test_first_known_answer_uses_prg_key_1():
    key, _, _ = known_answers()[0]
    assert oracle.prg_key(1) == key


def test_prg_keys_differ_only_in_last_byte():
    k1, k2, k3 = (oracle.prg_key(m) for m in (1, 2, 3))
    assert k1 == bytes(range(16))
    assert k2 == bytes(range(15)) + b"\x10"
    assert k3 == bytes(range(15)) + b"\x11"


def openssl_ecb(key: bytes, data: bytes) -> bytes:
    res = subprocess.run(["openssl", "enc", "-aes-128-ecb", "-nopad", "-K", key.hex()],
                         input=data, capture_output=True, check=True)
    return res.stdout


@pytest.mark.skipif(shutil.which("openssl") is None, reason="openssl command-line tool not present")
def test_aes_matches_openssl_on_random_blocks():
    rng = np.random.default_rng(197)
    keys = [oracle.prg_key(m) for m in (1, 2, 3)] + [rng.integers(0, 256, 16, dtype=np.uint8).tobytes() for _ in range(3)]
    for key in keys:
        blocks = rng.integers(0, 256, (64, 16), dtype=np.uint8)
        want = openssl_ecb(key, blocks.tobytes())
        got = b"".join(oracle.aes128_encrypt(key, b.tobytes()) for b in blocks)
        assert got == want


@pytest.mark.skipif(shutil.which("openssl") is None, reason="openssl command-line tool not present")
def test_prg_is_mmo_over_openssl_aes():
    """G_m(s) = E_{k_m}(s') xor s' with s' = s with the control bit cleared."""
    rng = np.random.default_rng(198)
    for m in (1, 2, 3):
        blocks = rng.integers(0, 256, (32, 16), dtype=np.uint8)
        cleared = blocks.copy()
        cleared[:, 0] &= 0xFE
        enc = np.frombuffer(openssl_ecb(oracle.prg_key(m), cleared.tobytes()), dtype=np.uint8).reshape(-1, 16)
        want = enc ^ cleared
        for b, w in zip(blocks, want):
            assert oracle.prg(m, b.tobytes()) == w.tobytes()


def test_prg_ignores_control_bit_of_its_input():
    rng = np.random.default_rng(199)
    for m in (1, 2, 3):
        b = bytearray(rng.integers(0, 256, 16, dtype=np.uint8).tobytes())
        b[0] &= 0xFE
        lo = oracle.prg(m, bytes(b))
        b[0] |= 1
        assert oracle.prg(m, bytes(b)) == lo


def test_aes_is_a_permutation_on_a_byte_slice():
    """Encrypting 256 blocks that differ in one byte gives 256 distinct outputs, and the
    all-zero key/plaintext value is the published one (FIPS-197 derived, OpenSSL-checked)."""
    key = bytes(16)
    outs = {oracle.aes128_encrypt(key, bytes([v]) + bytes(15)) for v in range(256)}
    assert len(outs) == 256
    assert oracle.aes128_encrypt(key, bytes(16)).hex() == "66e94bd4ef8a2c3b884cfa59ca342b2e"
