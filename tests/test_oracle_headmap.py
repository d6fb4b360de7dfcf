"""Pins for the oracle's Algorithm 1 (head mapping construction, Section 4.1)."""
import json
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_headmap_handworked_fixture():
    with open(os.path.join(GOLDEN, "headmap_handworked.json")) as f:
        case = json.load(f)
    a_t = np.array(case["a_t"], np.float32)[None, :, None, :]   # [S=1,Ht,R=1,N]
    a_d = np.array(case["a_d"], np.float32)[None, :, None, :]
    mp, ov = oracle.head_mapping(a_d, a_t, case["k"])
    np.testing.assert_array_equal(ov, case["overlap"])
    np.testing.assert_array_equal(mp, case["map"])


def test_headmap_overlap_sums_over_rows_and_samples_and_matches_sets():
    rng = np.random.default_rng(0)
    S, Hd, Ht, R, N, k = 3, 4, 6, 5, 40, 7
    a_d = rng.random((S, Hd, R, N), dtype=np.float32)
    a_t = rng.random((S, Ht, R, N), dtype=np.float32)
    mp, ov = oracle.head_mapping(a_d, a_t, k)
    want = np.zeros((Ht, Hd), np.int64)
    for s in range(S):
        for r in range(R):
            td = [set(np.argsort(-a_d[s, h, r], kind="stable")[:k]) for h in range(Hd)]
            for t in range(Ht):
                tt = set(np.argsort(-a_t[s, t, r], kind="stable")[:k])
                for h in range(Hd):
                    want[t, h] += len(tt & td[h])
    np.testing.assert_array_equal(ov, want)
    np.testing.assert_array_equal(mp, want.argmax(1))      # argmax returns the first maximum


def test_headmap_recovers_planted_permutation():
    rng = np.random.default_rng(1)
    S, Hd, R, N, k = 2, 5, 4, 64, 8
    a_d = rng.random((S, Hd, R, N), dtype=np.float32)
    src = np.array([3, 3, 0, 4, 1, 2, 2, 0])
    a_t = a_d[:, src] + 0.01 * rng.random((S, len(src), R, N), dtype=np.float32)
    mp, _ = oracle.head_mapping(a_d, a_t, k)
    np.testing.assert_array_equal(mp, src)
