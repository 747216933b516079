"""The library's engine and tile choice against recorded measurements (no GPU needed).

bs_choose_engine and bs_planes_tile are time models fitted on one machine (Sec. 4.1.1 / 4.2: the faster execution
method per layer).  tests/golden/engine_times_mi355x.txt holds the measured time of every engine and tile on 375
shapes; the choice must stay close to the fastest one on them, so that an edit of a coefficient or of the tile
rule that moves a boundary the wrong way fails here."""
import os

import numpy as np
import pytest

import paper_1709_04060_amd as bs

HERE = os.path.dirname(os.path.abspath(__file__))
U, TC, BP = bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT, bs.BS_BIPOLAR


def load():
    rows = []
    for line in open(os.path.join(HERE, "golden", "engine_times_mi355x.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        w, a, M, N, K = (int(x) for x in f[:5])
        t = {"bitserial": float(f[5]), "i8_256": float(f[6]), "i8_128": float(f[7]), "i8_64": float(f[8])}
        if f[9] != "-":
            t["fp4_256"], t["fp4_128"], t["fp4_64"] = float(f[9]), float(f[10]), float(f[11])
        rows.append((w, a, M, N, K, t))
    return rows


def chosen_time(w, a, M, N, K, t):
    wf = BP if w == 1 else TC
    af = BP if (w == 1 and a == 1) else U
    e = bs.bs_choose_engine(w, wf, a, af, M, N, K)
    if e == bs.BS_ENGINE_BITSERIAL:
        return t["bitserial"]
    tile = bs.bs_planes_tile(M, N)[0]
    return t[("fp4_%d" if e == bs.BS_ENGINE_DENSE_FP4 else "i8_%d") % tile]


def test_fixture_covers_the_fitted_range():
    rows = load()
    assert len(rows) == 375
    assert {(w, a) for w, a, *_ in rows} == {(1, 1), (1, 2), (2, 2), (3, 3), (4, 4)}
    assert all(("fp4_256" in t) == (max(w, a) <= 2) for w, a, _, _, _, t in rows)


def test_choice_is_close_to_the_fastest_engine_on_the_recorded_shapes():
    regret = np.array([chosen_time(*r) / min(r[5].values()) - 1.0 for r in load()])
    # as fitted: 0.4 % on average, 15 % at worst; the bounds leave room for a refit, not for a wrong boundary
    assert regret.mean() < 0.01, regret.mean()
    assert regret.max() < 0.20, regret.max()
    assert (regret > 0.10).sum() <= 8, (regret > 0.10).sum()


def test_a_single_engine_everywhere_is_far_worse():
    """What the choice buys: always bit-serial or always matrix cores lose a large factor somewhere."""
    rows = load()
    always_bs = np.array([r[5]["bitserial"] / min(r[5].values()) - 1.0 for r in rows])
    always_mc = np.array([min(v for k, v in r[5].items() if k != "bitserial") / min(r[5].values()) - 1.0 for r in rows])
    assert always_bs.mean() > 0.5 and always_bs.max() > 10
    assert always_mc.mean() > 0.5 and always_mc.max() > 3


def test_tile_rule_picks_the_faster_tile():
    """bs_planes_tile against the three measured tiles, per engine kind: within 10 % of the fastest tile on every
    recorded shape but a handful, never worse than 15 %."""
    loss = []
    for w, a, M, N, K, t in load():
        tile = bs.bs_planes_tile(M, N)[0]
        for kind in ("i8", "fp4"):
            if kind + "_256" in t:
                loss.append(t["%s_%d" % (kind, tile)] / min(t[kind + "_256"], t[kind + "_128"], t[kind + "_64"]) - 1.0)
    loss = np.array(loss)
    assert loss.max() < 0.15, loss.max()
    assert (loss > 0.10).mean() < 0.02, (loss > 0.10).mean()


@pytest.mark.parametrize("M,N,want", [(4096, 4096, 256), (256, 256, 64), (1024, 1024, 64), (1024, 2048, 64), (1536, 2048, 64),
                                      (2048, 2048, 128), (384, 10816, 128), (2048, 2176, 128), (2048, 4096, 128), (3072, 3072, 256), (8192, 8192, 256)])
def test_tile_rule_examples(M, N, want):
    tile, rounds, tiles = bs.bs_planes_tile(M, N)
    assert tile == want
    per = {256: 256, 128: 512, 64: 1024}[tile]  # workgroups of that tile the chip holds at a time
    assert tiles == -(-M // tile) * -(-N // tile) and rounds == -(-tiles // per)
