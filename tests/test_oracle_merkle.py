"""Pins for the oracle's Merkle commitment: the hash against published vectors and an independent program, the tree
against hand-expanded small cases and structural invariants, proofs against the root."""
import hashlib
import shutil
import subprocess

import numpy as np
import pytest

import synth
from oracle import verillm_oracle as O

RNG = np.random.default_rng(4242)


def H(b):
    return hashlib.sha256(b).digest()


def test_sha256_published_vectors():
    # FIPS 180 example messages: the empty string and "abc"
    assert hashlib.sha256(b"").hexdigest() == "e3b0c44298fc1c149afbf4c8996fb92427ae41e4649b934ca495991b7852b855"
    assert hashlib.sha256(b"abc").hexdigest() == "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"


@pytest.mark.skipif(shutil.which("sha256sum") is None, reason="coreutils sha256sum not installed")
def test_leaf_digest_equals_an_independent_program_on_the_serialised_bytes():
    x = np.array([1.0, -2.5, 3.0e-20, 0.0, -0.0], dtype=np.float32)
    leaves = O.merkle_leaves(x)
    # canonical serialization: IEEE-754 binary32, little endian; 1.0 = 00 00 80 3f, -0.0 = 00 00 00 80
    raw = [bytes([0x00, 0x00, 0x80, 0x3F]), bytes([0x00, 0x00, 0x20, 0xC0]), x[2:3].astype("<f4").tobytes(), bytes(4),
           bytes([0, 0, 0, 0x80])]
    for leaf, b in zip(leaves, raw):
        out = subprocess.run(["sha256sum"], input=b, capture_output=True, check=True).stdout.split()[0].decode()
        assert leaf.hex() == out
    assert leaves[3] != leaves[4]                        # +0 and -0 are different scalars on the wire


def test_tree_small_cases_written_out():
    x = RNG.standard_normal(7).astype(np.float32)
    l = O.merkle_leaves(x)
    assert O.merkle_root(x[:1]) == l[0]
    assert O.merkle_root(x[:2]) == H(l[0] + l[1])
    assert O.merkle_root(x[:3]) == H(H(l[0] + l[1]) + l[2])                       # the unpaired leaf moves up unchanged
    assert O.merkle_root(x[:4]) == H(H(l[0] + l[1]) + H(l[2] + l[3]))
    assert O.merkle_root(x[:5]) == H(H(H(l[0] + l[1]) + H(l[2] + l[3])) + l[4])
    assert O.merkle_root(x[:6]) == H(H(H(l[0] + l[1]) + H(l[2] + l[3])) + H(l[4] + l[5]))
    assert O.merkle_root(x[:7]) == H(H(H(l[0] + l[1]) + H(l[2] + l[3])) + H(H(l[4] + l[5]) + l[6]))


def test_tree_composes_from_aligned_halves_and_reacts_to_every_leaf():
    x = RNG.standard_normal(64).astype(np.float32)
    assert O.merkle_root(x) == H(O.merkle_root(x[:32]) + O.merkle_root(x[32:]))
    y = RNG.standard_normal(48).astype(np.float32)      # 48 = 32 + 16: the right part is a smaller complete tree moved up
    assert O.merkle_root(y) == H(O.merkle_root(y[:32]) + O.merkle_root(y[32:]))
    root = O.merkle_root(x)
    seen = {root}
    for j in range(64):
        z = x.copy()
        z[j] = np.nextafter(z[j], np.float32(np.inf))    # one unit in the last place
        r = O.merkle_root(z)
        assert r not in seen
        seen.add(r)
    assert O.merkle_root(x[::-1].copy()) != root          # order matters


def test_records_in_bf16_are_hashed_as_their_exact_float32_values():
    x = RNG.standard_normal(40).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    assert O.merkle_root(bits) == O.merkle_root(synth.bf16_bits_to_f32(bits))
    assert O.merkle_root(bits) != O.merkle_root(x)
    assert O.merkle_root(x.astype(np.float64)) == O.merkle_root(x)
    roots = O.merkle_roots(np.stack([x, x[::-1]]))
    assert roots.shape == (2, 32) and roots.dtype == np.uint8 and bytes(roots[0]) == O.merkle_root(x)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 13, 64, 100])
def test_every_opening_verifies_and_any_change_is_rejected(n):
    x = RNG.standard_normal(n).astype(np.float32)
    root = O.merkle_root(x)
    depth = max(n - 1, 0).bit_length()
    for j in range(n):
        path = O.merkle_open(x, j)
        assert len(path) <= depth
        assert O.merkle_verify(root, x[j], j, n, path)
        assert not O.merkle_verify(root, np.nextafter(x[j], np.float32(9)), j, n, path)      # another scalar
        if n > 1:
            assert not O.merkle_verify(root, x[j], (j + 1) % n, n, path) or x[j] == x[(j + 1) % n]
            bad = [bytes([path[0][0] ^ 1]) + path[0][1:]] + path[1:]
            assert not O.merkle_verify(root, x[j], j, n, bad)                              # a forged sibling
            assert not O.merkle_verify(root, x[j], j, n, path[:-1])                        # a truncated proof
            assert not O.merkle_verify(root, x[j], j, n, path + [path[-1]])                # a padded proof
    if n == 8:
        assert all(len(O.merkle_open(x, j)) == 3 for j in range(8))
    if n == 5:
        assert [len(O.merkle_open(x, j)) for j in range(5)] == [3, 3, 3, 3, 1]
