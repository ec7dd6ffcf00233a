"""Pin for the oracle's memory-shuffle copy (Section V-D): the slot-to-slot move of cached rows [0, len) for every
(layer, K|V, head), against the same move written with numpy slicing on the [L][2][C][nh][S][d] array -- every byte of
the cache compared, for 2- and 4-byte elements, including a move of no rows and a move of a full slot."""
import numpy as np
import pytest

from oracle import oracle as orc


@pytest.mark.parametrize("ebytes", [2, 4])
def test_compact_equals_numpy_slicing(ebytes):
    L, Cn, nh, S, d = 3, 9, 5, 37, 24          # no power of two anywhere: a wrong stride cannot hide
    rng = np.random.default_rng(11 + ebytes)
    dt = np.uint16 if ebytes == 2 else np.uint32
    cache = rng.integers(0, np.iinfo(dt).max, size=(L, 2, Cn, nh, S, d), dtype=dt)
    src, dst, ln = [8, 0, 6, 3], [1, 5, 2, 7], [S, 0, 1, 20]      # full slot, nothing, one row, a ragged piece
    want = cache.copy()
    for a, b, n in zip(src, dst, ln):
        want[:, :, b, :, :n, :] = cache[:, :, a, :, :n, :]
    got = cache.copy()
    orc.compact(got, L, Cn, nh, S, d, ebytes, src, dst, ln)
    assert np.array_equal(got, want)
    # what a move must leave alone: rows >= len of the destination, the sources, every slot not named
    assert np.array_equal(got[:, :, 7, :, 20:], cache[:, :, 7, :, 20:])
    assert np.array_equal(got[:, :, 5], cache[:, :, 5])               # the move of no rows changed nothing
    for s in (0, 3, 4, 6, 8):
        assert np.array_equal(got[:, :, s], cache[:, :, s])
    assert not np.array_equal(got[:, :, 1], cache[:, :, 1])           # and the full-slot move really happened


def test_compact_chain_applies_move_by_move():
    # moves are applied in list order: a slot vacated by an earlier move may be the target of a later one
    L, Cn, nh, S, d = 1, 4, 2, 6, 8
    cache = np.arange(L * 2 * Cn * nh * S * d, dtype=np.uint16).reshape(L, 2, Cn, nh, S, d)
    want = cache.copy()
    want[:, :, 0, :, :4] = cache[:, :, 1, :, :4]
    want[:, :, 1, :, :5] = cache[:, :, 3, :, :5]
    got = cache.copy()
    orc.compact(got, L, Cn, nh, S, d, 2, [1, 3], [0, 1], [4, 5])
    assert np.array_equal(got, want)


def test_server_shuffle_moves_exactly_the_cached_rows():
    """The same copy inside the fused run: after an eviction that forces a move, the moved request's K/V rows [0, len)
    read back from its new slot equal what its old slot held, for every layer, K and V, and head."""
    import dataclasses
    import flover_synth as synth
    cfg = dataclasses.replace(synth.tiny_gpt(), C=4, S=32)
    w = synth.make_weights(cfg, 3)
    srv = orc.OracleServer(cfg, w)
    rng = np.random.default_rng(5)
    for rid, (p, g) in enumerate(((3, 9), (4, 1), (5, 9), (6, 9))):
        srv.add_request(rid, rng.integers(0, cfg.V, size=p), g)
    srv.step(False)                                   # request 1 (slot 1) ends
    n = int(srv.state()["len"][3])
    before = {(l, kv, h): srv.read_kv(l, kv, 3, h, n) for l in range(cfg.L) for kv in (0, 1) for h in range(cfg.nh)}
    rr = srv.reorder_evict()
    assert rr.moves == [(3, 1)] and rr.bytes_moved == 2 * n * 2 * cfg.L * cfg.H * 4
    st = srv.state()
    assert int(st["req_id"][1]) == 3 and int(st["len"][1]) == n and st["state"][3] == 0
    for (l, kv, h), rows in before.items():
        assert np.array_equal(srv.read_kv(l, kv, 1, h, n), rows)
        assert np.abs(rows).max() > 0
    srv.close()
