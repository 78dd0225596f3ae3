"""Pins for the CPU oracle: each check ties one oracle function to something
other than the oracle itself -- a NumPy/torch library routine on a special
case, a closed form, a hand-worked value, brute force on tiny inputs, or the
LSH collision law of Section 2, eq. (3)."""
import math
import os

import numpy as np
import pytest


# --------------------------------------------------------------------------- hash, eq. (2)

def test_hash_equals_numpy_packbits(oracle):
    # special case that is a library routine: sign test of a matmul, little-endian bit packing
    rng = np.random.default_rng(11)
    for d, r in ((128, 16), (128, 32), (128, 64), (7, 5), (33, 40)):
        X = rng.standard_normal((50, d)).astype(np.float32)
        R = rng.standard_normal((d, r)).astype(np.float32)
        got = oracle.hash_codes(X, R)
        bits = (X.astype(np.float64) @ R.astype(np.float64)) >= 0
        W = (r + 31) // 32
        padded = np.zeros((50, W * 32), dtype=np.uint8)
        padded[:, :r] = bits
        want = np.packbits(padded, axis=1, bitorder="little").view("<u4").reshape(50, W)
        assert got.dtype == np.uint32 and got.shape == (50, W)
        np.testing.assert_array_equal(got, want)


def test_hash_hand_worked_signed_identity(oracle):
    # d = 3, hyperplanes +e0, -e1, +e2, +e0 (r = 4): bits are read off coordinate signs
    R = np.array([[1, 0, 0, 1],
                  [0, -1, 0, 0],
                  [0, 0, 1, 0]], dtype=np.float32)
    X = np.array([[2.0, 3.0, -1.0],     # bits: 1, 0, 0, 1  -> 0b1001 = 9
                  [-1.0, -5.0, 4.0],    # bits: 0, 1, 1, 0  -> 0b0110 = 6
                  [0.0, 0.0, 0.0],      # sgn(0) = 1 everywhere -> 0b1111 = 15
                  [-0.5, 0.0, 0.0]],    # bits: 0, 1 (-0.0 >= 0), 1, 0 -> 6
                 dtype=np.float32)
    np.testing.assert_array_equal(oracle.hash_codes(X, R)[:, 0], [9, 6, 15, 6])


def test_hash_invariants(oracle):
    rng = np.random.default_rng(5)
    d, r = 64, 40
    X = rng.standard_normal((200, d)).astype(np.float32)
    R = rng.standard_normal((d, r)).astype(np.float32)
    c = oracle.hash_codes(X, R)
    # positive scaling leaves the code unchanged
    np.testing.assert_array_equal(oracle.hash_codes(X * np.float32(37.5), R), c)
    # negation complements the low r bits (no projection is exactly zero here)
    mask = np.array([0xFFFFFFFF, (1 << (r - 32)) - 1], dtype=np.uint32)
    np.testing.assert_array_equal(oracle.hash_codes(-X, R), (~c) & mask)
    # unused high bits are zero
    assert np.all((c[:, 1] >> np.uint32(r - 32)) == 0)


def test_hash_margin_is_cosine(oracle):
    rng = np.random.default_rng(6)
    X = rng.standard_normal((20, 32)).astype(np.float32)
    R = rng.standard_normal((32, 9)).astype(np.float32)
    _, m = oracle.hash_codes(X, R, with_margin=True)
    Xd, Rd = X.astype(np.float64), R.astype(np.float64)
    want = np.abs(Xd @ Rd) / (np.linalg.norm(Xd, axis=1)[:, None] * np.linalg.norm(Rd, axis=0)[None, :])
    np.testing.assert_allclose(m, want, rtol=1e-12, atol=0)


@pytest.mark.parametrize("theta", [0.0, math.pi / 6, math.pi / 3, math.pi / 2,
                                   2 * math.pi / 3, math.pi])
def test_lsh_collision_law(oracle, theta):
    # eq. (3): E[d_H(h(x), h(y))] / r = theta / pi for two vectors at angle theta
    rng = np.random.default_rng(int(theta * 1000) + 1)
    d, r, pairs = 24, 64, 400
    dist = 0
    for _ in range(pairs // 50):
        R = rng.standard_normal((d, r)).astype(np.float32)
        a = rng.standard_normal((50, d))
        a /= np.linalg.norm(a, axis=1, keepdims=True)
        b = rng.standard_normal((50, d))
        b -= np.sum(a * b, axis=1, keepdims=True) * a
        b /= np.linalg.norm(b, axis=1, keepdims=True)
        x = a
        y = math.cos(theta) * a + math.sin(theta) * b
        # different norms on purpose: the law is about the angle only
        cx = oracle.hash_codes((3.0 * x).astype(np.float32), R)
        cy = oracle.hash_codes((0.25 * y).astype(np.float32), R)
        for i in range(50):
            dist += int(oracle.score(cx[i:i + 1], cy[i:i + 1])[0])
    n = pairs * r
    p = theta / math.pi
    if theta == 0.0:
        assert dist == 0
    elif theta == math.pi:
        assert dist == n
    else:
        sigma = math.sqrt(p * (1 - p) / n)
        assert abs(dist / n - p) < 4 * sigma


# --------------------------------------------------------------------------- score, eq. (5)

def test_score_brute_force_and_bounds(oracle):
    rng = np.random.default_rng(7)
    for W, G in ((1, 1), (1, 4), (2, 4), (2, 3)):
        codes = rng.integers(0, 2 ** 32, size=(300, W), dtype=np.uint64).astype(np.uint32)
        cq = rng.integers(0, 2 ** 32, size=(G, W), dtype=np.uint64).astype(np.uint32)
        got = oracle.score(codes, cq)
        want = np.zeros(300, dtype=np.int64)
        for s in range(300):
            for g in range(G):
                for w in range(W):
                    want[s] += bin(int(codes[s, w]) ^ int(cq[g, w])).count("1")
        np.testing.assert_array_equal(got, want)
        assert got.min() >= 0 and got.max() <= G * W * 32
        # library cross-check: unpackbits
        x = codes[:, None, :] ^ cq[None, :, :]
        np.testing.assert_array_equal(
            got, np.unpackbits(x.view(np.uint8), axis=-1).reshape(300, -1).sum(axis=1))


def test_score_identities(oracle):
    r = 20
    mask = np.uint32((1 << r) - 1)
    c = np.array([[0xABCDE & int(mask)]], dtype=np.uint32)
    assert oracle.score(c, c)[0] == 0
    assert oracle.score(c, (~c) & mask)[0] == r
    # three query heads that all see the complement: 3 r
    assert oracle.score(c, np.repeat((~c) & mask, 3, axis=0))[0] == 3 * r
    # symmetric in its two arguments
    a = np.array([[0x13579BDF]], dtype=np.uint32)
    b = np.array([[0x2468ACE0]], dtype=np.uint32)
    assert oracle.score(a, b)[0] == oracle.score(b, a)[0]


# --------------------------------------------------------------------------- select, eq. (6)

def test_select_hand_worked(oracle):
    pos = np.arange(6, dtype=np.int32)
    # largest Hamming distance wins (argmin of the negative distance)
    assert oracle.select([1, 3, 0, 2, 3, 1], pos, 6, t=6) == 1          # tie 1 vs 4 -> lowest
    assert oracle.select([0, 0, 0, 0, 0, 0], pos, 6, t=6) == 0          # all equal -> slot 0
    assert oracle.select([1, 2, 3, 4, 5, 9], pos, 6, t=6) == 5
    # not full: append at n_valid regardless of scores
    assert oracle.select([9, 9, 9, -1, -1, -1], pos, 3, t=3) == 3


def test_select_protects_sink_and_recent(oracle):
    # slots hold tokens 0,1,7,3,9,8 ; new token is t = 10
    pos = np.array([0, 1, 7, 3, 9, 8], dtype=np.int32)
    sc = np.array([9, 9, 5, 4, 9, 9], dtype=np.int32)
    assert oracle.select(sc, pos, 6, t=10) == 0
    # first two tokens are sinks -> slots 0, 1 protected; most recent 2 tokens (9, 8) protected
    assert oracle.select(sc, pos, 6, t=10, n_sink=2, n_recent=2) == 2
    # only recent protection
    assert oracle.select(sc, pos, 6, t=10, n_recent=2) == 0
    # recent = 3 also protects token 7
    assert oracle.select(sc, pos, 6, t=10, n_sink=2, n_recent=3) == 3


def test_evicted_slot_is_complement_code(oracle):
    # r = 4, C = 5: the slot holding the bitwise complement of the query code is the victim
    R = np.eye(4, dtype=np.float32)
    keys = np.array([[1, 1, 1, 1], [1, -1, 1, 1], [-1, -1, -1, -1], [1, 1, -1, 1], [-1, 1, 1, 1]],
                    dtype=np.float32)
    u = oracle.UnitCache(5, 4, 4, 1, R)
    for t in range(5):
        res = u.decode_step(keys[t:t + 1], keys[t], keys[t], t)
        assert res["evicted"] == t                       # filling: append
    np.testing.assert_array_equal(u.codes[:, 0], [15, 13, 0, 11, 14])
    res = u.decode_step(np.array([[1, 1, 1, 1]], dtype=np.float32),
                        np.array([1, 1, -1, -1], dtype=np.float32),
                        np.array([5, 6, 7, 8], dtype=np.float32), 5)
    np.testing.assert_array_equal(res["scores"], [0, 1, 4, 1, 1])
    assert res["evicted"] == 2
    np.testing.assert_array_equal(u.codes[:, 0], [15, 13, 3, 11, 14])
    np.testing.assert_array_equal(u.slot_pos, [0, 1, 5, 3, 4])
    np.testing.assert_array_equal(u.V[2], [5, 6, 7, 8])
    assert int(u.n_valid[0]) == 5


# --------------------------------------------------------------------------- attention, eq. (1)

def test_attend_closed_forms(oracle):
    rng = np.random.default_rng(3)
    d = 16
    q = rng.standard_normal((2, d)).astype(np.float32)
    V = rng.standard_normal((6, d)).astype(np.float32)
    # one slot: output is that value row
    np.testing.assert_allclose(oracle.attend(q, V[:1] * 0 + 1, V[:1]), np.stack([V[0], V[0]]),
                               rtol=1e-12)
    # all keys equal: uniform weights -> mean of V
    Keq = np.tile(rng.standard_normal((1, d)).astype(np.float32), (6, 1))
    np.testing.assert_allclose(oracle.attend(q, Keq, V),
                               np.tile(V.astype(np.float64).mean(0), (2, 1)), rtol=1e-12)
    # two slots, logits (a, 0) with the 1/sqrt(d) scale: d = 4, q = 2 e0, k0 = a e0 -> q.k/2 = a
    a = 1.25
    q2 = np.array([[2.0, 0, 0, 0]], dtype=np.float32)
    K2 = np.array([[a, 0, 0, 0], [0, 0, 0, 0]], dtype=np.float32)
    V2 = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]], dtype=np.float32)
    p0 = math.exp(a) / (math.exp(a) + 1.0)
    np.testing.assert_allclose(oracle.attend(q2, K2, V2)[0], [p0, 1 - p0, 0, 0], rtol=1e-12,
                               atol=1e-15)


def test_attend_equals_numpy_and_torch(oracle):
    import torch
    rng = np.random.default_rng(4)
    G, n, d = 4, 77, 128
    q = rng.standard_normal((G, d)).astype(np.float32)
    K = (rng.standard_normal((n, d)) * 2).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    got, prob = oracle.attend(q, K, V, with_prob=True)
    a = q.astype(np.float64) @ K.astype(np.float64).T / math.sqrt(d)
    a = np.exp(a - a.max(axis=1, keepdims=True))
    a /= a.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(prob, a, rtol=1e-12)
    np.testing.assert_allclose(got, a @ V.astype(np.float64), rtol=1e-11, atol=1e-13)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double()[None], torch.from_numpy(K).double()[None],
        torch.from_numpy(V).double()[None])[0].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)
    # occupied-slot count is honoured
    got5 = oracle.attend(q, K, V, n_valid=5)
    np.testing.assert_allclose(got5, oracle.attend(q, K[:5], V[:5]), rtol=0, atol=0)


# --------------------------------------------------------------------------- Algorithm 1

def _brute_force_policy(Kall, Vall, Qall, R, C, G, n_sink=0, n_recent=0):
    """Independent NumPy statement of the policy with fixed slots (tiny sizes only)."""
    N, d = Kall.shape
    r = R.shape[1]
    bits = lambda X: (X.astype(np.float64) @ R.astype(np.float64) >= 0).astype(np.int64)
    slot_tok = []
    log = []
    for t in range(N):
        if len(slot_tok) < C:
            slot_tok.append(t)
            log.append(len(slot_tok) - 1)
            continue
        hb = bits(Kall[slot_tok])                              # [C][r]
        qb = bits(Qall[:, t])                                  # [G][r]
        dist = np.zeros(C, dtype=np.int64)
        for g in range(G):
            dist += np.sum(hb != qb[g][None, :], axis=1)
        ok = np.array([(p >= n_sink) and (p <= t - 1 - n_recent) for p in slot_tok])
        dist_m = np.where(ok, dist, -1)
        e = int(np.argmax(dist_m))                             # first maximum = lowest slot
        slot_tok[e] = t
        log.append(e)
    return np.array(slot_tok), np.array(log)


@pytest.mark.parametrize("sink,recent", [(0, 0), (2, 3)])
def test_prefill_equals_brute_force(oracle, sink, recent):
    rng = np.random.default_rng(21)
    d, r, C, G, N = 8, 6, 12, 3, 90
    R = rng.standard_normal((d, r)).astype(np.float32)
    Kall = rng.standard_normal((N, d)).astype(np.float32)
    Vall = rng.standard_normal((N, d)).astype(np.float32)
    Qall = rng.standard_normal((G, N, d)).astype(np.float32)
    u = oracle.UnitCache(C, d, r, G, R, n_sink=sink, n_recent=recent)
    log = u.prefill(Kall, Vall, Qall)
    slot_tok, blog = _brute_force_policy(Kall, Vall, Qall, R, C, G, sink, recent)
    np.testing.assert_array_equal(u.slot_pos, slot_tok)
    np.testing.assert_array_equal(log, blog[C:])
    np.testing.assert_array_equal(u.K, Kall[slot_tok])
    np.testing.assert_array_equal(u.V, Vall[slot_tok])
    np.testing.assert_array_equal(u.codes, oracle.hash_codes(Kall[slot_tok], R))
    if sink:
        assert set(range(sink)) <= set(slot_tok.tolist())
        assert set(range(N - recent, N)) <= set(slot_tok.tolist())


def test_prefill_short_prompt_is_identity(oracle):
    rng = np.random.default_rng(22)
    d, r, C, G, N = 8, 6, 12, 2, 7
    R = rng.standard_normal((d, r)).astype(np.float32)
    Kall = rng.standard_normal((N, d)).astype(np.float32)
    Vall = rng.standard_normal((N, d)).astype(np.float32)
    Qall = rng.standard_normal((G, N, d)).astype(np.float32)
    u = oracle.UnitCache(C, d, r, G, R)
    assert len(u.prefill(Kall, Vall, Qall)) == 0
    assert int(u.n_valid[0]) == N
    np.testing.assert_array_equal(u.slot_pos, list(range(N)) + [-1] * (C - N))
    np.testing.assert_array_equal(u.K[:N], Kall)


def test_decode_trajectory_invariants(oracle):
    from paper_2412_16187_amd import synth
    w = synth.TOY.scaled(budget=24, n_prompt=16, n_decode=120, head_dim=32, hash_bits=12,
                         gqa_group=2)
    R = synth.projection(w)
    x = synth.gen_unit(w, 1)
    u = oracle.UnitCache(w.budget, w.head_dim, w.hash_bits, w.gqa_group, R)
    u.prefill(x["K"][:16], x["V"][:16], x["Q"][:, :16])
    assert int(u.n_valid[0]) == 16
    for t in range(16, 136):
        before = u.slot_pos.copy()
        nv = int(u.n_valid[0])
        res = u.decode_step(x["Q"][:, t], x["K"][t], x["V"][t], t)
        e = res["evicted"]
        # cache never exceeds the budget; exactly one slot changes; new token is kept
        assert int(u.n_valid[0]) == min(nv + 1, w.budget)
        changed = np.nonzero(before != u.slot_pos)[0]
        np.testing.assert_array_equal(changed, [e])
        assert u.slot_pos[e] == t
        if nv < w.budget:
            assert e == nv
        else:
            sc = res["scores"]
            assert sc[e] == sc.max() and e == int(np.argmax(sc))
        held = u.slot_pos[: int(u.n_valid[0])]
        assert len(set(held.tolist())) == len(held)
        # code table stays coherent with the key cache
        np.testing.assert_array_equal(u.codes[: len(held)], oracle.hash_codes(u.K[: len(held)], R))
        # attention is over the updated cache: the new token attends to itself
        want = oracle.attend(x["Q"][:, t], u.K, u.V, n_valid=len(held))
        np.testing.assert_array_equal(res["out"], want)


def test_codes_in_override_drives_the_step(oracle):
    # the lock-step harness may hand in codes; they must be the ones scored and stored
    R = np.eye(4, dtype=np.float32)
    u = oracle.UnitCache(2, 4, 4, 1, R)
    one = np.ones(4, dtype=np.float32)
    u.decode_step(one[None], one, one, 0)
    u.decode_step(one[None], -one, one, 1)           # codes: slot0 = 15, slot1 = 0
    res = u.decode_step(one[None], one, one, 2, codes_in=np.array([[0], [5]], dtype=np.uint32))
    np.testing.assert_array_equal(res["scores"], [4, 0])
    assert res["evicted"] == 0 and int(u.codes[0, 0]) == 5


def test_units_driver_matches_single_unit(oracle):
    rng = np.random.default_rng(9)
    U, C, d, r, G = 5, 10, 16, 8, 2
    R = rng.standard_normal((d, r)).astype(np.float32)
    units = [oracle.UnitCache(C, d, r, G, R) for _ in range(U)]
    K = np.zeros((U, C, d), np.float32); V = np.zeros((U, C, d), np.float32)
    codes = np.zeros((U, C, 1), np.uint32); pos = np.full((U, C), -1, np.int32)
    nv = np.zeros(U, np.int32)
    for t in range(25):
        q = rng.standard_normal((U, G, d)).astype(np.float32)
        k = rng.standard_normal((U, d)).astype(np.float32)
        v = rng.standard_normal((U, d)).astype(np.float32)
        out, ev = oracle.decode_step_units(K, V, codes, pos, nv, R, q, k, v,
                                           np.full(U, t, np.int32), G, r, n_threads=2)
        for i, u in enumerate(units):
            res = u.decode_step(q[i], k[i], v[i], t)
            assert res["evicted"] == ev[i]
            np.testing.assert_array_equal(res["out"], out[i])
            np.testing.assert_array_equal(u.slot_pos, pos[i])


# --------------------------------------------------------------------------- method sanity

def test_hash_eviction_loses_less_attention_than_random(oracle):
    # Section 4.8 defines attention loss as the attention mass of evicted tokens.  Direction
    # only: on peaked synthetic queries the policy must beat evicting a uniformly random slot.
    from paper_2412_16187_amd import synth
    w = synth.LLAMA8B_DECODE.scaled(n_prompt=192, budget=64, n_decode=64, hash_bits=32)
    R = synth.projection(w)
    rng = np.random.default_rng(0)
    loss_h, loss_r = [], []
    for unit in range(3):
        x = synth.gen_unit(w, unit)
        u = oracle.UnitCache(w.budget, w.head_dim, w.hash_bits, w.gqa_group, R)
        u.prefill(x["K"][:w.n_prompt], x["V"][:w.n_prompt], x["Q"][:, :w.n_prompt])
        rand_tok = list(range(w.budget))
        for t in range(w.budget, w.n_prompt):
            rand_tok[int(rng.integers(w.budget))] = t
        for t in range(w.n_prompt, w.n_prompt + w.n_decode):
            u.decode_step(x["Q"][:, t], x["K"][t], x["V"][t], t, attend=False)
            rand_tok[int(rng.integers(w.budget))] = t
            _, p = oracle.attend(x["Q"][:, t], x["K"][: t + 1], x["V"][: t + 1], with_prob=True)
            loss_h.append(1.0 - p[:, u.slot_pos].sum(axis=1).mean())
            loss_r.append(1.0 - p[:, rand_tok].sum(axis=1).mean())
    assert np.mean(loss_h) < np.mean(loss_r)


def test_needles_survive_prompt_compression(oracle):
    # Long-context recipe: a few prompt keys ("needles") that later queries point at.  Direction
    # only: after the prompt stage the share of needles still cached must exceed the share of
    # the prompt the budget keeps, i.e. the policy prefers them to an average token.
    from paper_2412_16187_amd import synth
    w = synth.LONG_CONTEXT.scaled(n_kv_heads=1, budget=300, n_prompt=1000, n_decode=0,
                                  needle_frac=0.03)
    R = synth.projection(w)
    kept, total = 0, 0
    for unit in range(4):
        x = synth.gen_unit(w, unit)
        u = oracle.UnitCache(w.budget, w.head_dim, w.hash_bits, w.gqa_group, R)
        u.prefill(x["K"][:w.n_prompt], x["V"][:w.n_prompt], x["Q"][:, :w.n_prompt])
        held = set(int(p) for p in u.slot_pos)
        kept += sum(int(p) in held for p in x["needle_pos"])
        total += len(x["needle_pos"])
    assert kept / total > w.budget / w.n_prompt, (kept, total)


# --------------------------------------------------------------------------- paper's worked figure

def test_hash_table_overhead_worked_example():
    # C*b bits per head (Section 3, Complexity); figures printed in Section 4.7
    path = os.path.join(os.path.dirname(__file__), "golden", "hash_table_overhead.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for layers, heads, batch, seq, frac, bits, mb in rows:
        slots = int(int(seq) * float(frac))
        total_bits = int(layers) * int(heads) * int(batch) * slots * int(bits)
        assert total_bits / 8 / 2 ** 20 == float(mb)


# --------------------------------------------------------------------------- L2-norm comparator

def test_l2_norm_definition(oracle):
    # exactly representable cases
    assert oracle.norm2(np.array([3, 4, 0, 0], np.float32)) == 25.0
    assert oracle.norm2(np.zeros(8, np.float32)) == 0.0
    # non-integer keys: the mathematical sum of squares, to double rounding (every square of a
    # float32 is exact in double; math.fsum adds them without error)
    rng = np.random.default_rng(1)
    for d in (5, 64, 128):
        x = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
        exact = math.fsum(float(v) * float(v) for v in x)
        assert abs(oracle.norm2(x) - exact) <= d * 2.0 ** -53 * exact
        np.testing.assert_allclose(oracle.norm2(x), np.dot(x.astype(np.float64), x.astype(np.float64)),
                                   rtol=1e-14)
    # 2^24 + 1 is not a float32: a single-precision sum would lose the 1
    assert oracle.norm2(np.array([4096, 1, 0, 0], np.float32)) == 16777217.0
    np.testing.assert_array_equal(oracle.norm2_rows(np.array([[1, 2], [0.5, 0]], np.float32)), [5.0, 0.25])


def _l2_brute_force(Kall, C, sink, recent, norm_of):
    """The comparator stated independently: slots hold token indices, the evictable slot with the
    largest norm (lowest slot on ties) takes each new token."""
    slot_tok, log = list(range(C)), []
    for t in range(C, len(Kall)):
        n2 = [norm_of(Kall[p]) for p in slot_tok]
        ok = [(p >= sink) and (p <= t - 1 - recent) for p in slot_tok]
        e = max((s for s in range(C) if ok[s]), key=lambda s: (n2[s], -s))
        slot_tok[e] = t
        log.append(e)
    return slot_tok, log


def test_l2_policy_evicts_largest_norm_brute_force(oracle):
    from fractions import Fraction
    rng = np.random.default_rng(2)
    for sink, recent in ((0, 0), (2, 3)):
        d, C, N = 6, 9, 60
        for integer_keys in (True, False):
            if integer_keys:   # every squared norm exact in any precision; many exact ties
                Kall = rng.integers(-3, 4, size=(N, d)).astype(np.float32)
                norm_of = lambda k: int(np.sum(k.astype(np.int64) ** 2))
            else:              # non-integer keys: exact rational arithmetic is the reference
                Kall = (rng.standard_normal((N, d)) * 3).astype(np.float32)
                norm_of = lambda k: sum(Fraction(float(v)) ** 2 for v in k)
            Vall = rng.standard_normal((N, d)).astype(np.float32)
            u = oracle.UnitCache(C, d, 8, 2, None, n_sink=sink, n_recent=recent, policy="l2")
            log = u.prefill(Kall, Vall, np.zeros((2, N, d), np.float32))
            slot_tok, blog = _l2_brute_force(Kall, C, sink, recent, norm_of)
            np.testing.assert_array_equal(log, blog)
            np.testing.assert_array_equal(u.slot_pos, slot_tok)
            np.testing.assert_array_equal(u.K, Kall[slot_tok])
            np.testing.assert_array_equal(u.V, Vall[slot_tok])
            np.testing.assert_allclose(u.norm2, [float(norm_of(Kall[p])) for p in slot_tok],
                                       rtol=0 if integer_keys else d * 2.0 ** -53)
            # a decode step: the victim is the largest norm; the new token attends to itself
            q = rng.standard_normal((2, d)).astype(np.float32)
            k = np.full(d, 100, np.float32)
            res = u.decode_step(q, k, k, N)
            e = res["evicted"]
            evictable = [s for s in range(C) if sink <= slot_tok[s] <= N - 1 - recent]
            assert e == max(evictable, key=lambda s: (res["norms"][s], -s))
            assert e == oracle.l2_select(res["norms"], slot_tok, C, N, sink, recent)
            np.testing.assert_array_equal(res["out"], oracle.attend(q, u.K, u.V))
            assert u.slot_pos[e] == N and u.norm2[e] == d * 100.0 ** 2


def test_l2_policy_decides_in_double(oracle):
    # slot 0 holds a key of squared norm 2^24, slot 1 one of 2^24 + 1: single precision cannot tell
    # them apart (and would evict slot 0 on the tie), the comparator's definition can
    d, C = 4, 3
    K = np.array([[4096, 0, 0, 0], [4096, 1, 0, 0], [1, 1, 1, 1], [2, 0, 0, 0]], np.float32)
    u = oracle.UnitCache(C, d, 8, 1, None, policy="l2")
    log = u.prefill(K, K, np.zeros((1, 4, d), np.float32))
    assert log.tolist() == [1]
    assert u.slot_pos.tolist() == [0, 3, 2]
    # a caller-supplied victim replaces the oracle's choice (the parity harness adopts the
    # device's victim in a near tie); its own choice is still what l2_select reports
    assert u.l2_select(4) == 0
    res = u.decode_step(np.zeros((1, d), np.float32), K[2], K[2], 4, victim_in=2)
    assert res["evicted"] == 2 and u.slot_pos.tolist() == [0, 3, 4] and u.norm2.tolist() == [2.0 ** 24, 4.0, 4.0]


def test_no_evictable_slot_is_rejected(oracle):
    import ctypes as C
    # a budget that the always-kept tokens fill completely is not a valid configuration
    with pytest.raises(ValueError):
        oracle.UnitCache(4, 8, 8, 1, np.zeros((8, 8), np.float32), n_sink=2, n_recent=2)
    for policy in ("hash", "l2"):
        with pytest.raises(ValueError):
            oracle.UnitCache(3, 8, 8, 1, np.zeros((8, 8), np.float32), n_sink=1, n_recent=3, policy=policy)
    # select reports -1 when every slot is protected, and apply then refuses to write
    assert oracle.select(np.array([5, 6, 7]), np.array([0, 1, 2]), 3, 3, n_sink=1, n_recent=2) == -1
    assert oracle.l2_select(np.array([5.0, 6, 7]), np.array([0, 1, 2]), 3, 3, n_sink=1, n_recent=2) == -1
    K = np.ones((3, 2), np.float32)
    V = K.copy()
    codes = np.full((3, 1), 9, np.uint32)
    spos = np.arange(3, dtype=np.int32)
    nv = np.array([3], np.int32)
    new = np.zeros(2, np.float32)
    c_new = np.zeros(1, np.uint32)
    f, u32, i32 = C.POINTER(C.c_float), C.POINTER(C.c_uint32), C.POINTER(C.c_int32)
    for e in (-1, 3):
        rc = oracle.lib().lsheo_apply(K.ctypes.data_as(f), V.ctypes.data_as(f), codes.ctypes.data_as(u32),
                                      spos.ctypes.data_as(i32), nv.ctypes.data_as(i32), 3, 2, 1, e,
                                      new.ctypes.data_as(f), new.ctypes.data_as(f),
                                      c_new.ctypes.data_as(u32), 7)
        assert rc == -1
        assert K.min() == 1 and V.min() == 1 and (codes == 9).all() and spos.tolist() == [0, 1, 2] and nv[0] == 3


# --------------------------------------------------------------------------- evicted attention mass

def test_evicted_mass_closed_form_and_numpy(oracle):
    # one cached key a*e0, new key 0, q = 2 e0, d = 4: logits (a, 0) -> mass on slot 0 = e^a / (e^a + 1)
    a = 0.75
    q = np.array([[2.0, 0, 0, 0]], np.float32)
    K = np.array([[a, 0, 0, 0]], np.float32)
    got = oracle.evicted_mass(q, K, np.zeros(4, np.float32), 0)
    np.testing.assert_allclose(got, [math.exp(a) / (math.exp(a) + 1)], rtol=1e-12)
    # independent float64 softmax over the C cached keys plus the new key
    rng = np.random.default_rng(8)
    G, C, d = 3, 17, 32
    q = rng.standard_normal((G, d)).astype(np.float32)
    K = rng.standard_normal((C, d)).astype(np.float32)
    k = rng.standard_normal(d).astype(np.float32)
    allk = np.concatenate([K, k[None]]).astype(np.float64)
    lg = q.astype(np.float64) @ allk.T / math.sqrt(d)
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    for e in (0, 5, 16):
        np.testing.assert_allclose(oracle.evicted_mass(q, K, k, e), p[:, e], rtol=1e-12)
    # masses over every possible victim plus the new token's own share sum to one
    tot = sum(oracle.evicted_mass(q, K, k, e) for e in range(C)) + p[:, C]
    np.testing.assert_allclose(tot, np.ones(G), rtol=1e-12)


def test_decode_step_reports_mass_of_its_victim(oracle):
    rng = np.random.default_rng(9)
    d, r, C, G = 16, 8, 6, 2
    R = rng.standard_normal((d, r)).astype(np.float32)
    for policy in ("hash", "l2"):
        u = oracle.UnitCache(C, d, r, G, R, policy=policy)
        for t in range(12):
            q = rng.standard_normal((G, d)).astype(np.float32)
            k = rng.standard_normal(d).astype(np.float32)
            Kold = u.K.copy()
            full = int(u.n_valid[0]) == C
            res = u.decode_step(q, k, k, t)
            if full:
                np.testing.assert_array_equal(res["mass"], oracle.evicted_mass(q, Kold, k, res["evicted"]))
                assert np.all(res["mass"] > 0) and np.all(res["mass"] < 1)
            else:
                assert not res["mass"].any()
