"""Host-side logic under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

tests/host_checks.cpp is built with g++ -fsanitize=address,undefined and linked with
 - the library's host-only integer code: the slice planner (csrc/p3_planner.h) and the
   run/tile arithmetic (csrc/p3_tiles.h), the same headers the gfx950 build compiles;
 - the CPU oracle (oracle/p3_oracle.cpp).
The driver works on exactly-sized heap buffers, so an access one element out of bounds,
a signed overflow or a misaligned access ends the run with a report (exit status != 0).
What it prints is checked here: the planner against the oracle's table and the
partition properties, the tile arithmetic against a brute-force partition in Python
(ragged runs, offsets beyond 2^31 elements), the sanitized oracle against the pins the
unsanitized one is held to.
"""
import os
import subprocess

import numpy as np
import pytest

from oracle import OraclePlan
from paper_1905_03960_amd import synthetic as sy

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "host_checks")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1905_03960_amd", "csrc"),
           "-o", exe, os.path.join(ROOT, "tests", "host_checks.cpp"), os.path.join(ROOT, "oracle", "p3_oracle.cpp")]
    subprocess.check_call(cmd)

    def run(lines):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0, f"sanitizer report or crash:\n{r.stderr[-4000:]}"
        out = r.stdout.splitlines()
        assert out and out[-1] == "end"
        assert not any(l.startswith("error") for l in out), [l for l in out if l.startswith("error")]
        return out[:-1]

    return run


def ints(line):
    return [int(x) for x in line.split()[1:]]


# ------------------------------------------------------------------ planner ----
@pytest.mark.parametrize("name,S", [("mlp", 50000), ("resnet50", 50000), ("vgg19", 50000), ("seq2seq", 50000),
                                    ("vgg19", 4096), ("vgg19", 4194304)])
def test_planner_equals_oracle_table_under_sanitizers(driver, name, S):
    sizes = sy.config(name)["layers"]
    out = driver([f"plan 1 0 {S} {len(sizes)} " + " ".join(map(str, sizes))])
    rc, K, N, arena, Kg = ints(out[0])
    o = OraclePlan(sizes, S)
    assert rc == 0 and K == o.K == Kg and N == o.N == sum(sizes) and arena >= N
    layer, off, ln = o.slice_table()
    rows = np.array([ints(l) for l in out[1:1 + K]], dtype=np.int64)
    lrows = np.array([ints(l) for l in out[1 + K:1 + K + len(sizes)]], dtype=np.int64)
    offsets = lrows[:, 3]
    assert (rows[:, 0] == layer).all() and (rows[:, 2] == ln).all() and (rows[:, 3] == np.arange(K)).all()
    assert (rows[:, 1] == offsets[layer] + off).all()                  # arena position = layer base + offset in layer
    assert (offsets % 64 == 0).all() and (np.diff(offsets) >= np.array(sizes[:-1])).all()
    assert (lrows[:, 2] == np.array(sizes)).all() and lrows[:, 1].sum() == K
    # tiles of the default size: what a brute-force count of touched grid cells gives
    cells = sum((s + n - 1) // 3328 - s // 3328 + 1 for s, n in zip(rows[:, 1].tolist(), rows[:, 2].tolist()))
    assert ints(out[-1]) == [cells]


def test_sharded_plans_partition_the_table_under_sanitizers(driver):
    sizes, S, G = [5, 50000, 50001, 99999, 100000, 100001, 7, 3], 10000, 3
    whole = driver([f"plan 1 0 {S} {len(sizes)} " + " ".join(map(str, sizes))])
    K = ints(whole[0])[1]
    all_rows = [tuple(ints(l)[:4]) for l in whole[1:1 + K]]
    seen = {}
    for j in range(G):
        out = driver([f"plan {G} {j} {S} {len(sizes)} " + " ".join(map(str, sizes))])
        rc, Kj, Nj, arena, Kg = ints(out[0])
        assert rc == 0 and Kg == K
        for l in out[1:1 + Kj]:
            layer, start, ln, gid = ints(l)[:4]
            assert gid % G == j and gid not in seen
            seen[gid] = (layer, start, ln, gid)
    assert [seen[g] for g in range(K)] == all_rows


def test_planner_refuses_bad_input_under_sanitizers(driver):
    out = driver(["plan 1 0 0 1 5", "plan 1 0 10 1 0", "plan 2 2 10 1 5", "plan 4 3 10 1 5",
                  f"plan 1 0 1 1 {2 ** 33}", f"plan 1 0 {2 ** 40} 1 {2 ** 35}", f"plan 1 0 {2 ** 20} 2 {2 ** 62} {2 ** 62}"])
    assert [ints(l)[0] for l in out] == [-1, -1, -1, -3, -3, -3, -3]


def test_first_step_handed_over_with_a_launch_is_the_oracles_order_cut_into_runs(driver):
    """The runs the host works out for the first selection step of a snapshot drain (they travel with the launch)
    against the oracle: the first `step` slices of the oracle's snapshot order for the same marks, cut where the
    layer changes or memory does not continue -- for random layer lists, mark subsets, step sizes and caps."""
    rng = np.random.default_rng(77)
    for case in range(120):
        L = int(rng.integers(1, 30))
        sizes = [int(max(1, round(10 ** rng.uniform(0, 5.3)))) for _ in range(L)]
        S = int(rng.choice([1, 7, 1000, 4096, 50000, 1 << 20])) if sum(sizes) < 30000 else int(rng.choice([1000, 4096, 50000]))
        step = int(rng.choice([1, 5, 64, 256, 832]))
        cap = int(rng.choice([1, 3, 16, 128]))
        marks = [int(x) for x in rng.permutation(L)[:int(rng.integers(1, L + 1))]]
        out = driver([f"first 1 0 {S} {step} {cap} {L} " + " ".join(map(str, sizes)) + f" {len(marks)} " +
                      " ".join(map(str, marks))])
        rc, n = ints(out[0])
        got = [tuple(ints(l)) for l in out[1:1 + n]]
        o = OraclePlan(sizes, S)
        layer, off, ln = o.slice_table()
        base = np.zeros(L, dtype=np.int64)              # the library's arena offsets: layers padded to 64 elements
        for l in range(1, L):
            base[l] = base[l - 1] + (sizes[l - 1] + 63) // 64 * 64
        order = o.order_snapshot(marks + [-1])[:step]
        want = []
        for i, g in enumerate(order):
            start = int(base[layer[g]] + off[g])
            if i > 0 and order[i - 1] + 1 == g and layer[g - 1] == layer[g]:
                want[-1][1] += int(ln[g])
            else:
                want.append([start, int(ln[g]), int(layer[g])])
        want = [tuple(w) for w in want][:cap]
        assert rc == 0 and got == want, (case, sizes, S, step, cap, marks, got[:4], want[:4])
    # nothing is handed over for an empty, a repeated or an unknown mark
    for bad in ("0", "2 1 1", "1 7"):
        out = driver([f"first 1 0 10 64 8 3 5 50 500 {bad}"])
        assert ints(out[0]) == [0, 0]


# ----------------------------------------------------------- tile arithmetic ----
def test_tiles_partition_their_run(driver):
    """Tiles of a run, in tile-number order, are consecutive, non-empty, cover the run exactly, lie within one
    grid cell each, and all but the first start on a cell boundary -- for ragged runs, offsets beyond 2^31
    elements and tile numbers near 2^32."""
    rng = np.random.default_rng(8)
    cases = []
    for i in range(300):
        tile = int(rng.choice([256, 3328, 4096, 1 << 20]))
        start = int(rng.integers(0, 2 ** 34)) if i % 3 else int(rng.integers(0, 5 * tile))
        ln = int(rng.integers(1, 40 * tile)) if i % 5 else int(rng.integers(1, 4))
        if i % 7 == 0:
            start -= start % tile                      # run that starts on a cell boundary
        if i % 11 == 0:
            ln = tile - start % tile                   # run that ends exactly on one
        tile0 = int(rng.integers(0, 2 ** 32 - 64 - ln // tile)) if i % 2 else int(rng.integers(0, 1000))
        cases.append((start, ln, i % 38, tile0, tile))
    out = driver([f"tiles {s} {n} {l} {t0} {t}" for s, n, l, t0, t in cases])
    at = 0
    for start, ln, layer, tile0, tile in cases:
        cells = ints(out[at])[0]
        assert cells == (start + ln - 1) // tile - start // tile + 1
        rows = [ints(l) for l in out[at + 1:at + 1 + cells]]
        at += 1 + cells
        pos = start
        for j, (ts, tn, tl) in enumerate(rows):
            assert ts == pos and 1 <= tn <= tile and tl == layer
            assert ts // tile == (ts + tn - 1) // tile                  # inside one cell
            assert j == 0 or ts % tile == 0
            pos += tn
        assert pos == start + ln
    assert at == len(out)


def test_run_records_that_could_become_wild_addresses_are_refused(driver):
    arena, L, tile = 5_000_000_000, 38, 3328
    start, ln = 3_000_000_123, 777_777
    cells = (start + ln - 1) // tile - start // tile + 1
    good = (start, ln, start % tile, 5, 1000, 1000 + cells)

    def rec(**kw):
        f = dict(zip(("start", "len", "grid_off", "layer", "tile0", "tile_end"), good))
        f.update(kw)
        return "valid {start} {len} {grid_off} {layer} {tile0} {tile_end} ".format(**f) + f"{arena} {L} {tile}"

    cmds = [rec(),
            rec(start=-8), rec(len=0), rec(len=-5), rec(start=arena - 10),            # leaves the arena
            rec(start=2 ** 62, len=2 ** 62),                                          # sum overflows
            rec(layer=L), rec(layer=-1),
            rec(grid_off=(start % tile) + 1), rec(grid_off=-1),
            rec(tile_end=1000 + cells + 1), rec(tile_end=1000 + cells - 1), rec(tile_end=1000), rec(tile_end=999),
            rec(tile0=999),                                                           # a stale numbering: one tile too many
            rec(start=arena - ln, grid_off=(arena - ln) % tile,
                tile_end=1000 + ((arena - 1) // tile - (arena - ln) // tile + 1))]    # ends exactly at the arena's end: fine
    got = [ints(l)[0] for l in driver(cmds)]
    assert got == [1] + [0] * 14 + [1]


# ------------------------------------------------- the oracle under sanitizers ----
def test_oracle_orders_under_sanitizers(driver, golden_dir):
    from test_oracle_order import brute_force_fifo, brute_force_ticked, read_golden
    g = read_golden(os.path.join(golden_dir, "three_layer_example.txt"))
    f = read_golden(os.path.join(golden_dir, "fifo_hand_cases.txt"))
    j = " ".join
    s = lambda xs: j(str(x) for x in xs)
    cmds = [f"oplan {g['slice_elems'][0]} 3 {s(g['layer_sizes'])}",
            f"oticked {s(g['release_ticks'])}", f"ofifo {s(g['release_ticks'])}",
            f"ofifo {s(f['a_release_ticks'])}", f"ofifo {s(f['b_release_ticks'])}",
            "osnap 4 2 1 0 -1", "osnap 6 2 -1 1 -1 0 -1",
            "oreplay 3 2 1 0 6 1 2 3 3 3 3", "oreplay 3 2 1 0 2 2 1"]
    out = [l for l in driver(cmds) if not l.startswith("o ")]          # without the oracle's slice rows
    assert ints(out[1])[1:] == g["p3_order"]
    assert ints(out[3])[1:] == g["fifo_order"]
    assert ints(out[5])[1:] == f["a_fifo_order"] and ints(out[6])[1:] == f["a_claim_ticks"]
    assert ints(out[7])[1:] == f["b_fifo_order"] and ints(out[8])[1:] == f["b_claim_ticks"]
    assert ints(out[9])[1:] == [0, 1, 2, 3, 4, 5]                       # all marked, one drain: identity
    assert ints(out[10])[1:] == [4, 5, 2, 3, 0, 1]                      # a drain per mark: backward order
    assert ints(out[11]) == [6] and ints(out[12])[1:] == [4, 2, 0, 1, 3, 5]
    assert ints(out[13])[0] < 0                                         # observed marks cannot decrease
    # random schedules against the set-based and the waiting-line brute force
    rng = np.random.default_rng(77)
    for _ in range(10):
        L = int(rng.integers(1, 9))
        sizes = [int(x) for x in rng.integers(1, 40, size=L)]
        S = int(rng.integers(1, 12))
        rel = [int(x) for x in rng.integers(0, 30, size=L)]
        out = [l for l in driver([f"oplan {S} {L} {s(sizes)}", f"oticked {s(rel)}", f"ofifo {s(rel)}"])
               if not l.startswith("o ")]
        assert ints(out[1])[1:] == brute_force_ticked(sizes, S, rel)
        want, ticks = brute_force_fifo(sizes, S, rel)
        assert ints(out[3])[1:] == want and ints(out[4])[1:] == ticks


@pytest.mark.parametrize("bf16", [False, True])
def test_oracle_arithmetic_under_sanitizers(driver, bf16):
    """Slices that end exactly at the end of the buffers (an overrun by one element would be reported), fp32 and
    bf16 copies; the result must equal the by-hand formula evaluated with numpy float32 operations."""
    sizes, S, W = [5, 1, 12, 7], 4, 3
    N = sum(sizes)
    cfg = dict(seed=31, W=W, dtype="bf16" if bf16 else "fp32", sigma_g=0.01, sigma_w=0.05, layers=sizes)
    grads, w0, _ = sy.make_inputs(cfg)
    m0 = sy.gaussian(32, 5, N, 0.01)
    lr, mu, rescale, wd = np.float32(0.1), np.float32(0.9), np.float32(0.5), np.float32(1e-3)
    o = OraclePlan(sizes, S)
    order = list(range(o.K))[::-1]
    words = []
    for g in grads:
        words += [f"{int(x):x}" for x in (g if bf16 else g.view(np.uint32))]
    words += [f"{int(x):x}" for x in w0.view(np.uint32)] + [f"{int(x):x}" for x in m0.view(np.uint32)]
    out = driver([f"oplan {S} {len(sizes)} " + " ".join(map(str, sizes)),
                  f"oapply {W} {1 if bf16 else 0} {float(lr)!r} {float(mu)!r} {float(rescale)!r} {float(wd)!r} "
                  f"{len(order)} " + " ".join(map(str, order)) + " " + " ".join(words)])
    K = ints(out[0])[0]
    assert ints(out[K + 1]) == [0]
    gw = np.array([int(x, 16) for x in out[K + 2].split()[1:]], dtype=np.uint32).view(np.float32)
    gm = np.array([int(x, 16) for x in out[K + 3].split()[1:]], dtype=np.uint32).view(np.float32)
    gs = [(g.astype(np.uint32) << 16).view(np.float32) if bf16 else g for g in grads]
    ssum = gs[0].copy()
    for g in gs[1:]:
        ssum = (ssum + g).astype(np.float32)
    ssum = (rescale * ssum).astype(np.float32)
    ssum = (ssum + (wd * w0).astype(np.float32)).astype(np.float32)
    m1 = ((mu * m0).astype(np.float32) - (lr * ssum).astype(np.float32)).astype(np.float32)
    w1 = (w0 + m1).astype(np.float32)
    assert (gm.view(np.uint32) == m1.view(np.uint32)).all() and (gw.view(np.uint32) == w1.view(np.uint32)).all()
