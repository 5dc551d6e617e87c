"""Pins for the oracle's projection (Sec. 3.1, Eq. 1, dense and restricted to I_t)."""
import os

import numpy as np

import oracle
from paper_2605_26444_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, V, d, M):
    W = synth.normal_bf16(seed, 0, (V, d), 0.02, threads=1)
    H = synth.normal_bf16(seed, 1, (M, d), 1.0, threads=1)
    return W, H


def test_worked_example():
    rows = {"W": [], "H": [], "Z": []}
    for line in open(os.path.join(GOLD, "head_worked_example.txt")):
        if line[0] in "WHZ" and line[1] == " ":
            rows[line[0]].append([float(x) for x in line[2:].split()])
    W = synth.f32_to_bf16_bits(np.array(rows["W"], np.float32))
    H = synth.f32_to_bf16_bits(np.array(rows["H"], np.float32))
    Z = np.array(rows["Z"])
    z32, z64 = oracle.head(W, H)
    assert np.array_equal(z64, Z) and np.array_equal(z32, Z.astype(np.float32))
    z32, z64 = oracle.head(W, H, ids=[2, 0])                      # restricted + reordered rows
    assert np.array_equal(z64, Z[:, [2, 0]])


def test_against_float64_matmul():
    """independent routine: numpy's float64 matmul of the decoded operands."""
    for seed, (V, d, M) in enumerate([(37, 24, 3), (200, 512, 5), (64, 1000, 1)]):
        W, H = rand_case(seed, V, d, M)
        Wf, Hf = synth.bf16_bits_to_f32(W).astype(np.float64), synth.bf16_bits_to_f32(H).astype(np.float64)
        ref = Hf @ Wf.T                                           # [M][V]
        z32, z64 = oracle.head(W, H)
        assert z64.shape == (M, V)
        assert np.allclose(z64, ref, rtol=1e-13, atol=1e-13)
        # products of two bf16 numbers are exact in fp32, so fp32 differs by accumulation only:
        # |fp32 - exact| <= gamma_d * sum |w h|, gamma_d ~ d * 2^-24
        bound = (d * 2.0 ** -24) * (np.abs(Hf) @ np.abs(Wf).T) * 1.01 + 1e-30
        assert np.all(np.abs(z32.astype(np.float64) - ref) <= bound)
        rng = np.random.default_rng(seed)
        ids = np.sort(rng.choice(V, size=V // 3, replace=False)).astype(np.int32)
        s32, s64 = oracle.head(W, H, ids=ids)
        assert np.allclose(s64, ref[:, ids], rtol=1e-13, atol=1e-13)


def test_unit_vector_reads_out_a_weight():
    V, d, M = 50, 64, 4
    W, _ = rand_case(5, V, d, M)
    cols = [0, 17, 63, 31]
    Hf = np.zeros((M, d), np.float32)
    for m, c in enumerate(cols):
        Hf[m, c] = 1.0
    z32, z64 = oracle.head(W, synth.f32_to_bf16_bits(Hf))
    Wf = synth.bf16_bits_to_f32(W)
    for m, c in enumerate(cols):
        assert np.array_equal(z32[m], Wf[:, c]) and np.array_equal(z64[m], Wf[:, c].astype(np.float64))


def test_sparse_equals_dense_restricted_bitwise():
    W, H = rand_case(9, 300, 256, 6)
    d32, d64 = oracle.head(W, H)
    ids = np.array([299, 0, 5, 5, 17, 123], np.int32)            # unsorted, with a duplicate
    s32, s64 = oracle.head(W, H, ids=ids)
    assert np.array_equal(s32, d32[:, ids]) and np.array_equal(s64, d64[:, ids])
    assert np.array_equal(s32[:, 2], s32[:, 3])                   # duplicated id -> identical logits
    # OpenMP build computes the same bits
    o32, o64 = oracle.head(W, H, ids=ids, omp=True)
    assert np.array_equal(o32, s32) and np.array_equal(o64, s64)


def test_bf16_round_trip_of_generator():
    x = np.array([1.0, 1.00390625, 1.01171875, -0.3, 3.0e38, 1e-40], np.float32)
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(b)
    assert back[0] == 1.0
    assert back[1] == 1.0            # 1 + 2^-8 is a tie between 1 and 1+2^-7: even mantissa wins
    assert back[2] == 1.015625       # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: rounds to even
    assert abs(back[3] + 0.3) < 0.3 * 2 ** -8
