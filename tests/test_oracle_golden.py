"""The oracle still reproduces the stored samples of the tiny configuration
(tests/golden/config0_oracle_samples.txt, written by tests/golden/make_golden.py)."""

import os

import numpy as np

from helpers import config0_oracle


def test_config0_oracle_matches_stored_samples():
    pre_out, dec_out, st = config0_oracle()
    path = os.path.join(os.path.dirname(__file__), "golden", "config0_oracle_samples.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        vals = np.array([float(x) for x in f[5:]])
        if f[0] == "prefill":
            li, b, i, j = map(int, f[1:5])
            got = pre_out[li][b, i, j, :4]
        else:
            t, li, b, j = map(int, f[1:5])
            got = dec_out[t][li][b, j, :4]
        np.testing.assert_allclose(got, vals, rtol=1e-13, atol=1e-14)
        n += 1
    assert n == 152
    # every sequence ends at 256 + 16 tokens in both caches
    assert st.seq_len(0, 0) == 272 and st.seq_len(1, 0) == 272
