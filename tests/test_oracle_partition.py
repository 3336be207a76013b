"""Pins for the oracle's block construction, partition and merge.

Each check is against something other than the oracle: the membership-mask
definition of Appendix A, NumPy fancy indexing, the closed-form parameter
counts of Section 2.1 / the footnote in Section 1, and invariants (disjoint
cover, no collisions, untouched unowned entries).
"""
import numpy as np
import pytest

import ist_inputs as gen
from oracle import ist_oracle as orc


def _cfg(dims, S, dtype="f32"):
    return gen.ISTConfig("t", 1, tuple(dims), S=S, B=4, k=1, rounds=1, dtype=dtype)


def _masks(perms, dims, S):
    """m[l][s] in {0,1}^{N_l}, built from the perm positions, not from oracle.block."""
    t = len(dims) - 1
    m = []
    for l in range(t + 1):
        if l == 0 or l == t:
            m.append(np.ones((S, dims[l]), dtype=np.int64))
        else:
            pos = np.empty(dims[l], dtype=np.int64)
            pos[perms[l - 1]] = np.arange(dims[l])
            # owner of perm position p: blocks as equal as N allows, the first N mod S one wider
            q, r = divmod(dims[l], S)
            owner = np.where(pos < r * (q + 1), pos // (q + 1), r + (pos - r * (q + 1)) // max(q, 1))
            m.append(np.stack([(owner == s).astype(np.int64) for s in range(S)]))
    return m


RAGGED = [((6, 8, 13, 5), 3), ((5, 11, 9, 7, 3), 5), ((7, 17, 4), 7), ((4, 10, 10, 3), 4), ((3, 7, 5, 2), 5)]


@pytest.mark.parametrize("dims,S", [((6, 8, 12, 5), 2), ((5, 12, 9, 6, 3), 3), ((7, 16, 4), 4),
                                    ((3, 5, 7, 2), 1)] + RAGGED)
def test_blocks_are_a_disjoint_cover(dims, S):
    cfg = _cfg(dims, S)
    perms = gen.make_perms(cfg)
    H = orc.blocks(perms, S)
    for l in range(1, cfg.t):
        allb = np.concatenate(H[l - 1])
        # sizes differ by at most one, the wider blocks first; equal when S divides N_l
        sizes = [len(h) for h in H[l - 1]]
        assert sum(sizes) == dims[l] and max(sizes) - min(sizes) <= 1 and sizes == sorted(sizes, reverse=True)
        if dims[l] % S == 0:
            assert all(n == dims[l] // S for n in sizes)
        # the same split as a library routine makes of the permutation
        for mine, ref in zip(H[l - 1], np.array_split(perms[l - 1], S)):
            assert np.array_equal(mine, ref)
        assert np.array_equal(np.sort(allb), np.arange(dims[l]))   # each neuron exactly once
    m = _masks(perms, dims, S)
    for l in range(cfg.t + 1):
        want = S if l in (0, cfg.t) else 1                         # sum_s m^{(s)}_{l,i}
        assert np.all(m[l].sum(axis=0) == want)
        if 0 < l < cfg.t:
            for s in range(S):
                assert np.array_equal(np.flatnonzero(m[l][s]), np.sort(H[l - 1][s]))


def test_block_of_an_indivisible_width():
    """10 neurons over 3 subnets: 4 + 3 + 3, in permutation order; out-of-range subnets are rejected."""
    perm = np.array([7, 2, 9, 0, 4, 1, 8, 3, 6, 5], dtype=np.int32)
    assert orc.block(perm, 3, 0).tolist() == [7, 2, 9, 0]
    assert orc.block(perm, 3, 1).tolist() == [4, 1, 8]
    assert orc.block(perm, 3, 2).tolist() == [3, 6, 5]
    assert orc.block(perm, 10, 9).tolist() == [5]
    with pytest.raises(ValueError):
        orc.block(perm, 3, 3)
    with pytest.raises(ValueError):
        orc.block(perm, 0, 0)


@pytest.mark.parametrize("dims,S", [((6, 8, 12, 5), 2), ((5, 12, 9, 6, 3), 3), ((7, 16, 4), 4)] + RAGGED)
def test_partition_equals_masked_definition_and_numpy(dims, S):
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.3)
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    H = orc.blocks(perms, S)
    m = _masks(perms, dims, S)
    t = cfg.t
    for s in range(S):
        for l in range(1, t + 1):
            rows = np.arange(dims[l]) if l == t else H[l - 1][s]
            cols = np.arange(dims[l - 1]) if l == 1 else H[l - 2][s]
            # (i) library routine as an independent opinion
            assert np.array_equal(subs[s][0][l - 1], Ws[l - 1][np.ix_(rows, cols)])
            # (ii) embedding the block in zeros equals (m_l m_{l-1}^T) * W_l
            emb = np.zeros_like(Ws[l - 1])
            emb[np.ix_(rows, cols)] = subs[s][0][l - 1]
            assert np.array_equal(emb, np.outer(m[l][s], m[l - 1][s]) * Ws[l - 1])
            assert np.array_equal(subs[s][1][l - 1], bs[l - 1][rows])


def test_parameter_counts_match_closed_form():
    dims, S = (6, 8, 12, 16, 5), 4
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg)
    subs = orc.partition(Ws, bs, gen.make_perms(cfg), S)
    t = cfg.t
    closed = dims[0] * dims[1] // S + sum(dims[i - 1] * dims[i] // S ** 2 for i in range(2, t)) \
        + dims[t - 1] * dims[t] // S
    full = sum(dims[i - 1] * dims[i] for i in range(1, t + 1))
    for s in range(S):
        assert sum(w.size for w in subs[s][0]) == closed
    assert full / S ** 2 <= closed <= full / S
    # the benchmark table: parameters per subnet of the five workloads
    want = {"cfg1": 8832, "cfg2": 2132992, "cfg3": 4204544, "cfg4": 168591360, "cfg5": 103168000}
    for name in want:
        c = gen.CONFIGS[name]
        d, S_ = c.dims, c.S
        p = d[0] * d[1] // S_ + sum(d[i - 1] * d[i] // S_ ** 2 for i in range(2, c.t)) \
            + d[c.t - 1] * d[c.t] // S_
        assert p == want[name]


@pytest.mark.parametrize("dims,S", RAGGED)
def test_parameter_counts_with_unequal_blocks(dims, S):
    """With N_l = q_l S + r_l the subnets hold, over all s, N_0 N_1 + N_{t-1} N_t first- and last-layer
    weights and, per middle matrix, sum_s w_l^s w_{l-1}^s = S q_l q_{l-1} + q_l r_{l-1} + q_{l-1} r_l +
    min(r_l, r_{l-1}) weights (the wider blocks are the first ones in both layers)."""
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg)
    subs = orc.partition(Ws, bs, gen.make_perms(cfg), S)
    t = cfg.t
    for l in range(1, t + 1):
        got = sum(subs[s][0][l - 1].size for s in range(S))
        if l == 1 or l == t:
            assert got == dims[l] * dims[l - 1]
        else:
            (q1, r1), (q0, r0) = divmod(dims[l], S), divmod(dims[l - 1], S)
            assert got == S * q1 * q0 + q1 * r0 + q0 * r1 + min(r1, r0)
        for s in range(S):
            rows = dims[l] if l == t else dims[l] // S + (s < dims[l] % S)
            cols = dims[l - 1] if l == 1 else dims[l - 1] // S + (s < dims[l - 1] % S)
            assert subs[s][0][l - 1].shape == (rows, cols) and subs[s][1][l - 1].shape == (rows,)


@pytest.mark.parametrize("dims,S", RAGGED)
def test_round_trip_and_unowned_entries_with_unequal_blocks(dims, S):
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.2)
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    parts = [np.array_split(p, S) for p in perms]             # a library routine's split of the permutation
    full = [np.full_like(w, 7.0) for w in Ws]
    orc.merge(full, None, perms, S, subs)
    for l in range(1, cfg.t + 1):
        owned = np.zeros(Ws[l - 1].shape, bool)
        for s in range(S):
            rows = np.arange(dims[l]) if l == cfg.t else parts[l - 1][s]
            cols = np.arange(dims[l - 1]) if l == 1 else parts[l - 2][s]
            assert not owned[np.ix_(rows, cols)].any()        # no collisions
            owned[np.ix_(rows, cols)] = True
        assert np.array_equal(full[l - 1][owned], Ws[l - 1][owned]) and np.all(full[l - 1][~owned] == 7.0)
    # hidden biases return to their neuron
    fb = [np.full_like(b, 7.0) for b in bs]
    orc.merge([w.copy() for w in Ws], fb, perms, S, subs)
    for l in range(cfg.t - 1):
        assert np.array_equal(fb[l], bs[l])


def test_single_hidden_layer_owns_every_weight():
    dims, S = (7, 16, 4), 4
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg)
    subs = orc.partition(Ws, bs, gen.make_perms(cfg), S)
    assert sum(w.size for s in range(S) for w in subs[s][0]) == sum(w.size for w in Ws)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merge_of_partition_is_identity_bitwise(dtype):
    dims, S = (5, 12, 8, 6, 3), 2
    cfg = _cfg(dims, S, dtype)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.2)
    if dtype == "bf16":
        Ws = [gen.to_bf16_bits(w).reshape(w.shape) for w in Ws]      # raw 2-byte elements
        bs_raw = [gen.to_bf16_bits(b) for b in bs]
        W0 = [w.copy() for w in Ws]
        subs = orc.partition(Ws, bs_raw, gen.make_perms(cfg), S)
        for w in Ws:
            w[...] = 0xFFFF
        # weights only: merge() averages the float output bias, checked elsewhere
        orc.merge(Ws, None, gen.make_perms(cfg), S, subs)
        H = orc.blocks(gen.make_perms(cfg), S)
        owned = [np.zeros(w.shape, bool) for w in Ws]
        for s in range(S):
            for l in range(1, cfg.t + 1):
                rows = np.arange(dims[l]) if l == cfg.t else H[l - 1][s]
                cols = np.arange(dims[l - 1]) if l == 1 else H[l - 2][s]
                owned[l - 1][np.ix_(rows, cols)] = True
        for w, w0, ow in zip(Ws, W0, owned):
            assert np.array_equal(w[ow], w0[ow]) and np.all(w[~ow] == 0xFFFF)
        return
    W0 = [w.copy() for w in Ws]
    b0 = [b.copy() for b in bs]
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    orc.merge(Ws, bs, perms, S, subs)
    for a, b in zip(Ws + bs, W0 + b0):
        assert a.tobytes() == b.tobytes()


def test_merge_leaves_unowned_entries_and_never_collides():
    dims, S = (5, 12, 8, 6, 3), 2
    cfg = _cfg(dims, S)
    Ws, bs = gen.make_weights(cfg)
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    # distinct markers per subnet element; count how often each target is written
    hits = [np.zeros(w.shape, dtype=np.float32) for w in Ws]
    ones = [([np.ones_like(w) for w in Wl], bl) for Wl, bl in subs]
    H = orc.blocks(perms, S)
    for s in range(S):
        for l in range(1, cfg.t + 1):
            ridx = None if l == cfg.t else H[l - 1][s]
            cidx = None if l == 1 else H[l - 2][s]
            tmp = np.zeros_like(hits[l - 1])
            orc.scatter(tmp, ridx, cidx, ones[s][0][l - 1])
            hits[l - 1] += tmp
    for l in range(1, cfg.t + 1):
        assert hits[l - 1].max() == 1.0                              # no position written twice
        unowned = int((hits[l - 1] == 0).sum())
        middle = 1 < l < cfg.t
        assert unowned == (dims[l] * dims[l - 1] * (S - 1) // S if middle else 0)
    # after a merge of modified subnets the unowned entries keep their bits
    W0 = [w.copy() for w in Ws]
    mod = [([w + 1.0 for w in Wl], bl) for Wl, bl in subs]
    orc.merge(Ws, bs, perms, S, mod)
    for l in range(cfg.t):
        un = hits[l] == 0
        assert np.array_equal(Ws[l][un], W0[l][un])
        assert np.array_equal(Ws[l][~un], W0[l][~un] + 1.0)


def test_output_bias_merge_is_the_mean():
    S, n = 4, 5
    rng = np.random.default_rng(0)
    b = rng.standard_normal((S, n)).astype(np.float32)
    cfg = _cfg((3, 8, n), S)
    Ws, bs = gen.make_weights(cfg)
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    subs = [(Wl, [bl[0], b[s]]) for s, (Wl, bl) in enumerate(subs)]
    orc.merge(Ws, bs, perms, S, subs)
    np.testing.assert_allclose(bs[-1], b.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
    # identical copies come back exactly when S is a power of two
    same = [(Wl, [bl[0], b[0]]) for Wl, bl in subs]
    orc.merge(Ws, bs, perms, S, same)
    assert np.array_equal(bs[-1], b[0])


def _merge_bias(b):
    """Output bias the oracle's merge produces from per-subnet copies b [S][n] (float32)."""
    S, n = b.shape
    cfg = _cfg((3, 2 * S, n), S)
    Ws, bs = gen.make_weights(cfg)
    perms = gen.make_perms(cfg)
    subs = orc.partition(Ws, bs, perms, S)
    subs = [(Wl, [bl[0], b[s]]) for s, (Wl, bl) in enumerate(subs)]
    orc.merge(Ws, bs, perms, S, subs)
    return bs[-1].astype(np.float32)


@pytest.mark.parametrize("S", [2, 8, 16, 64, 128])
def test_output_bias_round_trip_is_exact_for_power_of_two_S(S):
    """merge(partition(b_t)) == b_t bit for bit: with identical copies every addition of the
    pairwise tree doubles its operand and the final scaling by 1/S is a power of two.  (A running
    sum x, 2x, 3x, ... would round at 3x.)"""
    rng = np.random.default_rng(S)
    x = rng.standard_normal(3000).astype(np.float32)
    got = _merge_bias(np.tile(x, (S, 1)))
    assert np.array_equal(got.view(np.uint32), x.view(np.uint32))


def test_output_bias_tree_shape_for_ragged_S():
    """The order of the binary32 additions, written out by hand for S = 3, 5, 6, 7."""
    f = np.float32
    rng = np.random.default_rng(11)
    for S in (3, 5, 6, 7):
        b = (rng.standard_normal((S, 400)) * 10.0 ** rng.integers(-3, 4, (S, 400))).astype(np.float32)
        v = [b[s] for s in range(S)]
        if S == 3:
            tot = (v[0] + v[1]) + v[2]
        elif S == 5:
            tot = ((v[0] + v[1]) + (v[2] + v[3])) + v[4]
        elif S == 6:
            tot = ((v[0] + v[1]) + (v[2] + v[3])) + (v[4] + v[5])
        else:
            tot = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + v[6])
        want = (tot * (f(1.0) / f(S))).astype(np.float32)
        assert np.array_equal(_merge_bias(b).view(np.uint32), want.view(np.uint32)), S
