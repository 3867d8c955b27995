"""Pins of oracle/perf_model.py to the numbers and rules the paper prints.  CPU only."""
import json
import os

import pytest

from oracle import perf_model as pm

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.json")))


def test_phi_reproduces_quoted_numbers():
    # M*N*K = 1024^3 with M = N (Fig. 2 caption): K = 1024 -> M = N = 1024, tile size 256.
    assert int(pm.phi(256, 256, 1024)) == G["phi_K1024_tile256"]["value"]
    assert round(pm.phi(256, 256, 1)) == G["phi_K1_tile256"]["value"]
    # the printed expression does not give them (the discrepancy that phi() resolves)
    assert round(pm.phi_printed(256, 256, 1024)) == 205 and round(pm.phi_printed(256, 256, 1)) == 1
    # closed-form special case: cubic tile T=K -> 2T^3 / 3T^2
    assert pm.phi(96, 96, 96) == pytest.approx(2 * 96 / 3)


def test_search_space_size():
    assert len(pm.deep_tilings()) == G["deep_tilings"]["value"]
    assert len(set(pm.deep_tilings())) == 24 and "mhnk" in pm.deep_tilings()
    assert len(pm.flat_tilings()) == G["flat_tilings"]["value"]
    assert pm.n_candidates(1024, 1024, 512, 512) == G["n_candidates_M1024_N1024_K512_H512"]["value"]


def test_rule3_discards_what_the_paper_says():
    """Sec. III-C on the example M = N = 1024, K = H = 512: of the multiples of 16, Rule 3 keeps only
    the tile sizes that divide their (power-of-two) dimension, i.e. discards 99 % of the choices."""
    dims = (1024, 1024, 512, 512)
    kept = 1
    for d in dims:
        ok = [t for t in range(16, d + 1, 16) if pm.padding_ok(d, t)]
        assert ok == [t for t in (16, 32, 64, 128, 256, 512, 1024) if t <= d]     # the divisors, nothing else
        kept *= len(ok)
    total = pm.n_candidates(*dims) // (len(pm.deep_tilings()) + len(pm.flat_tilings()))
    assert kept == 7 * 7 * 6 * 6
    assert 1.0 - kept / total >= G["rule3_discard_fraction_min"]["value"]
    # a dimension that is not a power of two: padding below 5 % is allowed (S8: M = 768)
    assert pm.padding_ok(768, 256) and pm.padding_ok(768, 128) and not pm.padding_ok(768, 512)
    assert pm.padding_ok(1000, 32) and not pm.padding_ok(1000, 96)   # 1024/1000 - 1 = 2.4 %; 1056/1000 - 1 = 5.6 %


def test_hoisting_factors_of_mhnk():
    ext = {"m": 8, "h": 3, "n": 5, "k": 4}
    # default association: every statement of C_C in m,h,n,k; those of C_E in m,h,n
    assert pm.trips("mhnk", "C_C", ext) == 8 * 3 * 5 * 4
    assert pm.trips("mhnk", "C_E", ext) == 8 * 3 * 5
    assert pm.trips("mhnk", "L_A", ext, hoist=False) == 8 * 3 * 5 * 4
    assert pm.trips("mhnk", "S_E", ext, hoist=False) == 8 * 3 * 5
    # S_E moved to the scope of h: saves the extent of the loop it leaves
    assert pm.trips("mhnk", "S_E", ext) == 8 * 3
    # L_A stays under k while k > 1 ...
    assert pm.trips("mhnk", "L_A", ext) == 8 * 3 * 5 * 4
    # ... and is governed by m alone once k has extent 1: a factor h*n fewer loads
    ext1 = dict(ext, k=1)
    before = pm.trips("mhnk", "L_A", ext1, drop_unit_loops=False)
    after = pm.trips("mhnk", "L_A", ext1)
    assert after == 8 and before == after * ext["h"] * ext["n"]
    # L_B is indexed by k and n: always innermost in mhnk; L_D sits at n
    assert pm.trips("mhnk", "L_B", ext) == 8 * 3 * 5 * 4
    assert pm.trips("mhnk", "L_D", ext) == 8 * 3 * 5
    # mhnk and mnkh with h of extent 1 move the same data (same per-block expression nk)
    ext2 = dict(ext1, h=1)
    for s in ("L_A", "L_B", "L_D", "S_E", "C_C", "C_E"):
        assert pm.trips("mhnk", s, ext2) == pm.trips("mnkh", s, ext2)


def test_eq1_shared_memory_and_rule3():
    tiles = {"m": 64, "n": 32, "k": 16, "h": 48}
    assert pm.shm_estm(tiles) == 64 * 16 + 16 * 32 + 64 * 32 + 32 * 48 + 64 * 48
    assert pm.shm_estm(tiles, "BD") == 16 * 32 + 32 * 48
    assert pm.padding_ok(1024, 128) and not pm.padding_ok(1024, 96)       # power of two: no padding
    assert pm.padding_ok(1000, 128) and not pm.padding_ok(768, 512)       # 2.4 % ok, 33 % not
    assert pm.padding_ok(80, 16) and not pm.padding_ok(80, 32)


def test_eq2_to_5_hand_evaluated():
    # dims 512/512/64/64, tiles 64 everywhere, one batch, 2-byte elements, W = 1e12 B/s,
    # P = 1e14 FLOP/s, 100 compute units.  Extents: m = n = 8, k = h = 1.
    dims = {"m": 512, "n": 512, "k": 64, "h": 64}
    tiles = {"m": 64, "n": 64, "k": 64, "h": 64}
    r = pm.estimate("mhnk", dims, tiles, batch=1, elem_bytes=2, W=1e12, P=1e14, n_units=100)
    assert r["mem_bytes"] == {"L_A": 65536, "L_B": 524288, "L_D": 524288, "S_E": 65536}
    assert r["model_bytes"] == 1179648 and r["compulsory_bytes"] == 2 * (3 * 512 * 64 + 64 * 512)
    assert r["flops"] == 67108864 and r["n_block"] == 8
    assert r["t_mem"] == pytest.approx(1.179648e-6, rel=1e-15)
    assert r["t_comp"] == pytest.approx(6.7108864e-7, rel=1e-15)
    assert r["alpha"] == 13.5
    assert r["t_estm"] == pytest.approx(2.498494464e-5, rel=1e-12)
    # whole-problem tiles: one block, compulsory traffic only, alpha = 101
    one = pm.estimate("mhnk", dims, dims, batch=1, elem_bytes=2, W=1e12, P=1e14, n_units=100)
    assert one["model_bytes"] == one["compulsory_bytes"] and one["alpha"] == 101
    # split bandwidths: re-read bytes charged at the faster level
    s = pm.estimate("mhnk", dims, tiles, 1, 2, W=1e12, P=1e14, n_units=100, W_reread=4e12)
    assert s["t_mem"] == pytest.approx(262144 / 1e12 + (1179648 - 262144) / 4e12, rel=1e-15)


def test_block_loops_keep_their_statements():
    """Sec. III-B removes loops of extent 1 and re-hoists; read here so that no statement leaves
    the loops bound to the block index (m, h, batch), because blocks share no on-chip memory.
    Hand-evaluated: dims M=256 N=128 K=32 H=64, tiles 64/128/32/32, batch 3, 2-byte elements:
    extents m=4, n=1, k=1, h=2 -> 24 blocks, each loading its A tile (64x32), the whole B
    (32x128), its D tile (128x32), computing C (64x128 over K=32) and E (64x32 over N=128) and
    storing its E tile (64x32).  (Without the reading L_B would run once, L_A and C_C 4 times.)"""
    dims = {"m": 256, "n": 128, "k": 32, "h": 64}
    tiles = {"m": 64, "n": 128, "k": 32, "h": 32}
    r = pm.estimate("mhnk", dims, tiles, batch=3, elem_bytes=2, W=1e12, P=1e14, n_units=100)
    assert r["n_block"] == 24
    assert r["mem_bytes"] == {"L_A": 24 * 64 * 32 * 2, "L_B": 24 * 32 * 128 * 2, "L_D": 24 * 128 * 32 * 2,
                              "S_E": 24 * 64 * 32 * 2}
    assert r["mem_bytes"] == {"L_A": 98304, "L_B": 196608, "L_D": 196608, "S_E": 98304}
    assert r["model_bytes"] == 589824 and r["compulsory_bytes"] == 221184
    assert r["flops"] == 24 * (2 * 64 * 128 * 32 + 2 * 64 * 128 * 32) == 25165824
    assert r["alpha"] == pytest.approx(124 / 24, rel=1e-15)
    assert r["t_estm"] == pytest.approx(4.34765824e-6, rel=1e-12)
    # the same through trips(): the block loops hold L_B although k and n are dead
    ext = pm.extents_of(dims, tiles)
    assert pm.trips("mhnk", "L_B", ext, block_loops="mh") == 8 and pm.trips("mhnk", "L_B", ext) == 1
    assert pm.trips("mhnk", "L_A", ext, block_loops="mh") == 8 and pm.trips("mhnk", "L_A", ext) == 4
    # T_N = N, T_K = K with one h tile (the case of the five evaluated workloads when N fits a tile)
    one_h = pm.estimate("mhnk", dims, dict(tiles, h=64), batch=3, elem_bytes=2, W=1e12, P=1e14, n_units=100)
    assert one_h["mem_bytes"]["L_B"] == 12 * 32 * 128 * 2 and one_h["mem_bytes"]["L_D"] == 12 * 128 * 64 * 2


def test_alpha_in_rounds():
    """eq. (5) for blocks that run in rounds: hand-evaluated values, the cases where it is 1, its
    relation to the printed form (never above it, equal to it only in the limit of one block
    more than whole rounds), and the same estimate() otherwise."""
    assert pm.alpha_rounds(256, 256) == 1.0 and pm.alpha_rounds(1024, 256) == 1.0     # whole rounds: nothing idle
    assert pm.alpha_rounds(384, 256) == pytest.approx(512 / 384)                      # 2 rounds, the second half empty
    assert pm.alpha_rounds(192, 256) == pytest.approx(256 / 192)                      # 1 round, a quarter of the units idle
    assert pm.alpha_rounds(257, 256) == pytest.approx(512 / 257)
    assert pm.alpha_rounds(32, 256) == 8.0
    for nb in (1, 7, 255, 256, 257, 511, 512, 513, 5000):
        for nu in (1, 64, 256, 1024):
            a, printed = pm.alpha_rounds(nb, nu), (nb + nu) / nb
            assert 1.0 <= a <= printed
            assert (a == 1.0) == (nb % nu == 0)
    # one block more than whole rounds approaches the printed form from below
    assert pm.alpha_rounds(256 * 50 + 1, 256) == pytest.approx((256 * 51) / (256 * 50 + 1))
    assert (256 * 50 + 1 + 256) / (256 * 50 + 1) - pm.alpha_rounds(256 * 50 + 1, 256) < 1e-4
    dims = {"m": 512, "n": 512, "k": 64, "h": 64}
    tiles = {"m": 128, "n": 64, "k": 64, "h": 64}
    a = pm.estimate("mhnk", dims, tiles, 96, 2, W=8e12, P=2.5e15, n_units=256)
    b = pm.estimate("mhnk", dims, tiles, 96, 2, W=8e12, P=2.5e15, n_units=256, rounds=True)
    assert a["n_block"] == b["n_block"] == 384 and a["alpha"] == pytest.approx(640 / 384) and b["alpha"] == pytest.approx(512 / 384)
    assert b["t_estm"] == pytest.approx((b["t_mem"] + b["t_comp"]) * 512 / 384)
    assert (a["t_mem"], a["t_comp"]) == (b["t_mem"], b["t_comp"])
