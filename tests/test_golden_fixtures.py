"""Hand-worked fixtures under tests/golden/ against the oracle (both of its halves)."""
import os

import numpy as np

from oracle import Oracle, OracleConfig, attend_definition

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _parse(path):
    out = {"visible": {}}
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, rest = line.split(None, 1) if " " in line else (line, "")
        if key == "visible":
            i, js = rest.split(":")
            out["visible"][int(i)] = [int(x) for x in js.split()]
        elif key.endswith(":"):
            out[key[:-1]] = [int(x) for x in rest.split()]
        elif key == "g":
            out["g"] = np.array([float(x) for x in rest.split()], np.float32)
        else:
            out[key] = float(rest)
    return out


def test_vertical_slash_mask_and_cache_state_by_hand():
    fx = _parse(os.path.join(GOLDEN, "vertical_slash_mask_w2.txt"))
    W, tau, g = int(fx["W"]), fx["tau"], fx["g"]
    n = len(g)
    # definition half: one-hot values turn the attention output into the weights, zero keys make them uniform
    K = np.zeros((n, 1, n), np.float32)
    V = np.eye(n, dtype=np.float32)[:, None, :]
    Q = np.zeros((n, 1, n), np.float32)
    out = attend_definition(K, V, g[:, None], Q, np.arange(n), W, tau, 1.0)
    for i in range(n):
        vis = fx["visible"][i]
        want = np.zeros(n)
        want[vis] = 1.0 / len(vis)
        assert np.allclose(out[i, 0], want, atol=1e-15), i
    # mechanism half, one token at a time
    o = Oracle(OracleConfig(1, 1, 1, n, 2, W, 1, 8, 16, True))
    promoted = []
    for p in range(n):
        _, prom = o.push_tokens(0, [0], [1], K[p:p + 1], V[p:p + 1], g[p:p + 1, None], tau)
        if prom[0, 0]:
            promoted.append(p)
    assert promoted == fx["promoted_at_push"]
    assert list(o.global_pos(0, 0, 0)) == fx["global_after"]
    _, _, _, ring_pos = o.head_tables(0, 0, 0)
    assert sorted(int(x) for x in ring_pos if x >= 0) == fx["ring_after"]
    # and what the cache then shows the next query is row 5 of the table
    got = o.attend_cached(0, 0, np.zeros((1, n), np.float32), 1.0)[0]
    want = np.zeros(n)
    want[fx["visible"][n - 1]] = 1.0 / len(fx["visible"][n - 1])
    assert np.allclose(got, want, atol=1e-15)
