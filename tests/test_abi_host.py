"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, rejects bad
arguments before touching the GPU, and builds launch plans that cover the operator's definition
(section 3.1: each kept query row attends the kept rows of its own segment, per branch).
No GPU needed: nothing here launches a kernel."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2403_09195_amd import binding, build
    if not os.path.exists(build.LIB_PATH):
        build.build()
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(B):
    raw = ctypes.CDLL(os.path.join(ROOT, "paper_2403_09195_amd", "libdfa.so"))
    for fname, names in (("dfa.h", B.EXPORTS), ("dfa_bench.h", B.BENCH_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared = set(re.findall(r"\b(dfa_[a-z_]+)\s*\(", header))
        assert declared == set(names), fname
        for name in declared:
            assert hasattr(raw, name), name
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["dfa.h", "dfa_bench.h"]
    assert B.version() >= 200
    for code in range(0, -9, -1):
        assert B.error_string(code) != "unknown error code"
    assert B.error_string(-99) == "unknown error code"


def test_host_index_map_matches_eq1_by_hand(B):
    # N = 16, w = 8, r = 2 (worked by hand from Eq. 1; head start h mod r)
    assert B.index_map(16, 3, 8, 2) == [[0, 2, 4, 6, 8, 10, 12, 14], [1, 3, 5, 7, 9, 11, 13, 15],
                                        [0, 2, 4, 6, 8, 10, 12, 14]]
    assert B.index_map(12, 2, 6, 3, head_offsets=[2, 1]) == [[2, 5, 8, 11], [1, 4, 7, 10]]
    assert B.index_map(8, 1, 8, 1) == [list(range(8))]


def _fwd_rc(mod, **kw):
    """dfa_forward return code with fake (never dereferenced) pointers."""
    a = dict(q=0x10000, k=0x20000, v=0x30000, out=0x40000, lse=0x50000, Bsz=1, H=2, N=64, D=64, dt=0,
             scale=0.125, branches=[(16, 2)], offs=None, sq=None)
    a.update(kw)
    st = a["sq"] or mod.Strides(a["N"] * a["H"] * 64, a["H"] * 64, 64)
    br, nb = mod._branches(a["branches"])
    if "nb" in kw:
        nb = kw["nb"]
    vp = ctypes.c_void_p
    return mod.lib().dfa_forward(vp(a["q"]), vp(a["k"]), vp(a["v"]), st, st, st, a["Bsz"], a["H"], a["N"], a["D"],
                               a["dt"], ctypes.c_float(a["scale"]), br, nb, mod._i32_array(a["offs"]),
                               vp(a["out"]), vp(a["lse"]), vp(a.get("ws")), ctypes.c_size_t(a.get("ws_bytes", 0)), None)


def test_forward_rejects_bad_arguments_before_any_gpu_work(B):
    assert _fwd_rc(B, q=None) == -1
    assert _fwd_rc(B, out=None) == -1
    assert _fwd_rc(B, D=128) == -2
    assert _fwd_rc(B, Bsz=0) == -2
    assert _fwd_rc(B, branches=[(16, 0)]) == -2          # r < 1
    assert _fwd_rc(B, branches=[(0, 1)]) == -2           # w < 1
    assert _fwd_rc(B, offs=[[0, 2]]) == -2               # offset outside [0, r)
    assert _fwd_rc(B, scale=0.0) == -2
    assert _fwd_rc(B, scale=float("nan")) == -2
    assert _fwd_rc(B, nb=0) == -3
    assert _fwd_rc(B, branches=[(16, 1)] * 9) == -3
    assert _fwd_rc(B, dt=7) == -4
    assert _fwd_rc(B, q=0x10004) == -5
    assert _fwd_rc(B, ws=0x60004, ws_bytes=1 << 20) == -5   # misaligned workspace
    assert _fwd_rc(B, sq=B.Strides(64 * 2 * 64, 2 * 64 + 4, 64)) == -5


def test_workspace_bytes_follows_the_split_rule(B):
    """Room for the partial results of a split launch, one block of 256 rows (out in fp16, then lse and a row scale in fp32) per workgroup:
    the single-image workload has 192 tiles of 16, 24 or 32 steps for 512 workgroup slots, and the longest walks
    are shared out until every slot has a workgroup; the batch of 16 fills the chip and needs none.  (Without a
    device the library assumes the MI355X's 256 compute units.)"""
    wl = [(1024, 1), (2048, 2), (4096, 4)]
    assert B.workspace_bytes(1, 12, 4096, 64, B.DFA_BF16, wl) == 512 * 256 * (64 * 2 + 8)
    assert B.workspace_bytes(16, 12, 4096, 64, B.DFA_BF16, wl) == 0
    assert B.workspace_bytes(1, 12, 4096, 64, B.DFA_F32, wl) == 0
    assert B.workspace_bytes(1, 12, 4096, 128, B.DFA_BF16, wl) == 0          # D the library does not take
    assert B.workspace_bytes(1, 12, 4096, 64, B.DFA_BF16, [(1024, 0)]) == 0   # r < 1
    # walks too short to share (a share would have fewer than 8 steps of 64 keys): no split however few the tiles
    assert B.workspace_bytes(1, 2, 512, 64, B.DFA_BF16, [(512, 1)]) == 0


def test_stage_entry_points_reject_bad_arguments_before_any_gpu_work(B):
    """dfa_gather / dfa_scatter / dfa_merge: argument errors are found on the host (fake, aligned pointers)."""
    L, vp, fake = B.lib(), ctypes.c_void_p, 0x10000
    st = B.Strides(64 * 2 * 64, 2 * 64, 64)

    def gather(x=fake, xg=fake, Bsz=1, H=2, N=64, D=64, dt=0, br=(16, 2), offs=None):
        return L.dfa_gather(vp(x), st, Bsz, H, N, D, dt, B.Branch(*br), B._i32_array(offs), vp(xg), None)

    def scatter(og=fake, out=fake, Bsz=1, H=2, N=64, D=64, dt=0, br=(16, 2), offs=None):
        return L.dfa_scatter(vp(og), Bsz, H, N, D, dt, B.Branch(*br), B._i32_array(offs), vp(out), None)

    def merge(ob=fake, lb=fake, nb=2, Bsz=1, H=2, N=64, D=64, dt=0, out=fake, lse=fake):
        return L.dfa_merge(vp(ob), vp(lb), nb, Bsz, H, N, D, dt, vp(out), vp(lse), None)

    assert gather(x=None) == -1 and gather(xg=None) == -1
    assert gather(D=32) == -2 and gather(br=(48, 2)) == -2 and gather(br=(16, 3)) == -2
    assert gather(offs=[0, 2]) == -2
    assert gather(dt=5) == -4
    assert gather(x=0x10008) == -5
    assert gather(Bsz=70000) == -7                           # b rides on a grid dimension
    assert scatter(og=None) == -1 and scatter(out=None) == -1
    assert scatter(br=(128, 1)) == -2 and scatter(dt=9) == -4 and scatter(out=0x10004) == -5
    assert scatter(H=70000, br=(16, 1)) == -7
    assert merge(ob=None) == -1 and merge(out=None) == -1
    assert merge(nb=0) == -3 and merge(nb=9) == -3
    assert merge(D=128) == -2 and merge(dt=3) == -4 and merge(ob=0x10004) == -5
    assert merge(N=1 << 22, H=64) == -7                      # one image no longer fits 32-bit counters


def test_stack_static_and_dense_entry_points_reject_bad_arguments_before_any_gpu_work(B):
    """dfa_encoder_stack checks every argument before its first launch (so an error never leaves a workspace half
    written); dfa_forward_static and dfa_dense_unfused likewise.  Fake, aligned pointers: every case here is refused."""
    L, vp, fake = B.lib(), ctypes.c_void_p, 0x10000

    def stack(layers=2, Bsz=1, H=2, N=256, D=64, scale=0.125, branches=((64, 1),), offs=None, x=fake, ws=None, ws_bytes=0, nb=None):
        br, n = B._branches(list(branches))
        return L.dfa_encoder_stack(vp(x), vp(fake), vp(fake), layers, Bsz, H, N, D, ctypes.c_float(scale), br,
                                   n if nb is None else nb, B._i32_array(offs), vp(fake), vp(fake), vp(fake), vp(ws),
                                   ctypes.c_size_t(ws_bytes), None)

    assert stack(x=None) == -1
    assert stack(layers=0) == -2 and stack(D=32) == -2
    assert stack(N=200) == -2                                  # B * N is no multiple of the 256-row tile
    assert stack(H=3) == -2                                    # embed 192 is no multiple of 128
    assert stack(branches=((64, 0),)) == -2                    # r < 1: found before the first projection is enqueued
    assert stack(offs=[[0, 1]]) == -2                          # offset outside [0, r)
    assert stack(scale=-1.0) == -2 and stack(scale=float("inf")) == -2
    assert stack(nb=0) == -3
    assert stack(x=0x10004) == -5 and stack(ws=0x20008, ws_bytes=1 << 20) == -5

    st = B.Strides(64 * 2 * 64, 2 * 64, 64)
    br, nb = B._branches([(16, 2)])

    def static(q=fake, out=fake, D=64, dt=0, scale=0.125, nbr=nb):
        return L.dfa_forward_static(vp(q), vp(fake), vp(fake), st, st, st, 1, 2, 64, D, dt, ctypes.c_float(scale), br, nbr,
                                    None, vp(out), vp(fake), None)

    assert static(q=None) == -1 and static(out=None) == -1
    assert static(D=128) == -2 and static(scale=0.0) == -2 and static(nbr=9) == -3 and static(dt=4) == -4
    assert static(q=0x10002) == -5

    def dense(q=fake, N=256, D=64, scale=0.125, ws=fake, ws_bytes=1 << 30, Bsz=1, H=2):
        s2 = B.Strides(N * H * 64, H * 64, 64)
        return L.dfa_dense_unfused(vp(q), vp(fake), vp(fake), s2, s2, s2, Bsz, H, N, D, ctypes.c_float(scale), vp(fake),
                                   vp(fake), vp(ws), ctypes.c_size_t(ws_bytes), None)

    assert dense(q=None) == -1 and dense(ws=None) == -1
    assert dense(N=200) == -2 and dense(N=8192) == -2 and dense(D=32) == -2 and dense(scale=0.0) == -2
    assert dense(q=0x10008) == -5
    assert dense(ws_bytes=1024) == B.DFA_ERR_WORKSPACE
    assert L.dfa_dense_unfused_workspace_bytes(2, 3, 256, 64) == 2 * 3 * 256 * 256 * 2 + 2 * 3 * 256 * 64 * 2
    assert L.dfa_dense_unfused_workspace_bytes(2, 3, 256, 32) == 0


def _expected_multiset(N, h, n, branches, offs):
    """(how often each token is a key of row n, the plain list of (first key, stride, count, 1)), from the
    definition: one visit per branch that keeps both n and the key in the same part."""
    counts = np.zeros(N, dtype=np.int32)
    plain = []
    for x, (w, r) in enumerate(branches):
        o = (h % r) if offs is None else offs[x][h]
        first = (n // w) * w + o
        if n >= first and (n - first) % r == 0:
            end = min(N, (n // w + 1) * w)
            counts[first:end:r] += 1
            plain.append((first, r, len(range(first, end, r)), 1))
    return counts, plain


def _check_tile_list(N, got, counts, plain):
    """The tile's progressions add up to the definition's multiset; they are either the plain per-branch list or a
    coalesced one: disjoint progressions, each of one multiplicity, in fewer 64-key steps than the plain list."""
    mine = np.zeros(N, dtype=np.int32)
    visits = np.zeros(N, dtype=np.int32)
    for (first, stride, count, mult) in got:
        assert count >= 1 and stride >= 1 and mult >= 1 and 0 <= first and first + stride * (count - 1) < N
        mine[first:first + stride * count:stride] += mult
        visits[first:first + stride * count:stride] += 1
    assert np.array_equal(mine, counts)
    if sorted(got) != sorted(plain):
        assert visits.max() == 1
        steps = lambda lst: sum((c + 63) // 64 for (_, _, c, _) in lst)
        assert steps(got) < steps(plain) and len(got) <= 32


@pytest.mark.parametrize("Bsz,H,N,branches,offs", [
    (1, 1, 256, [(64, 2)], None),
    (1, 12, 4096, [(1024, 1), (2048, 2), (4096, 4)], None),
    (16, 12, 4096, [(1024, 1), (2048, 2), (4096, 4)], None),
    (2, 3, 16384, [(2048, 1), (4096, 2), (8192, 4), (16384, 8)], None),
    (3, 4, 360, [(120, 3), (180, 2), (360, 5)], [[2, 0, 1, 2], [1, 1, 0, 0], [4, 3, 0, 1]]),
    (40, 2, 96, [(32, 4), (96, 1)], None),
    # ragged partitions: w does not divide N, w > N, r does not divide w, a last part of one token
    (2, 3, 50, [(16, 3), (7, 2), (64, 5)], None),
    (1, 2, 1025, [(1024, 1), (300, 7)], [[0, 0], [6, 2]]),
    # the same branch twice: every key counts double
    (1, 2, 512, [(256, 2), (256, 2), (512, 1)], None),
])
def test_plan_covers_the_definition(B, Bsz, H, N, branches, offs):
    p = B.plan_describe(Bsz, H, N, branches, offs)
    tiles, rows, segs, items = p["tiles"], p["rows"], p["segs"], p["items"]
    seen = np.zeros((H, N), dtype=np.int32)
    total_pairs = 0
    for (h, rb, nr, sb, ns, _) in tiles:
        assert 1 <= nr <= 256
        tile_rows = rows[rb:rb + nr]
        seen[h, tile_rows] += 1
        got = [tuple(int(x) for x in segs[s]) for s in range(sb, sb + ns)]
        for n in (tile_rows if N <= 4096 else tile_rows[[0, -1]]):
            counts, plain = _expected_multiset(N, h, int(n), branches, offs)
            _check_tile_list(N, got, counts, plain)
        total_pairs += nr * sum(c * m for (_, _, c, m) in got)
    assert np.all(seen == 1)                                    # every (h, n) in exactly one tile
    assert len(items) % 8 == 0
    real = items[items[:, 0] >= 0]
    pairs = set(map(tuple, real.tolist()))
    assert len(pairs) == len(real) == len(tiles) * Bsz          # every (tile, b) launched once
    assert real[:, 1].min() == 0 and real[:, 1].max() == Bsz - 1
    if all(N % w == 0 and w % r == 0 for (w, r) in branches):
        assert total_pairs == H * sum(N * w // (r * r) for (w, r) in branches)   # N*w/r^2 pairs per branch


def test_plan_visits_a_key_of_several_branches_once(B):
    """The workload's nested branches (offsets h mod r): a row of all three branches has 3072 (query, key) pairs
    but only 2048 distinct keys, a row of the first two 2048 and 1536; the plan walks the distinct ones."""
    N, H, branches = 4096, 12, [(1024, 1), (2048, 2), (4096, 4)]
    p = B.plan_describe(1, H, N, branches)
    visited = 0
    for (h, rb, nr, sb, ns, _) in p["tiles"]:
        lst = p["segs"][sb:sb + ns]
        n = int(p["rows"][rb])
        member = [n % r == h % r for (_, r) in branches]
        distinct = int(lst[:, 2].sum())
        assert distinct == {1: 1024, 2: 1536, 3: 2048}[sum(member)]
        assert int(lst[:, 3].max()) == sum(member)
        visited += nr * distinct
    assert visited == H * (2048 * 1024 + 1024 * 1536 + 1024 * 2048)


def test_plan_keeps_a_unit_on_one_die_when_there_are_enough_units(B):
    # workgroup i runs on die i mod 8; all tiles of one (b, h) should share a die (and its L2)
    p = B.plan_describe(16, 12, 4096, [(1024, 1), (2048, 2), (4096, 4)])
    die_of = {}
    for i, (t, b) in enumerate(p["items"]):
        if t < 0:
            continue
        unit = (int(b), int(p["tiles"][t][0]))
        die_of.setdefault(unit, set()).add(i % 8)
    assert len(die_of) == 16 * 12
    assert all(len(d) == 1 for d in die_of.values())
    per_die = np.bincount([next(iter(d)) for d in die_of.values()], minlength=8)
    assert per_die.min() == per_die.max() == 24


def test_plan_runs_the_tiles_of_a_unit_together_on_long_lists(B):
    """Throughput workload: 384 items per die.  Outside the last 96 items of a die's list (which go heaviest
    first) the 16 tiles of a (b, h) unit follow one another, heaviest first."""
    p = B.plan_describe(16, 12, 4096, [(1024, 1), (2048, 2), (4096, 4)])
    items, tiles = p["items"], p["tiles"]
    for die in range(8):
        lst = [(int(t), int(b)) for (t, b) in items[die::8] if t >= 0]
        assert len(lst) == 384
        body, tail = lst[:-96], lst[-96:]
        units = [(b, int(tiles[t][0])) for (t, b) in body]
        for lo in range(0, len(body), 16):
            assert len(set(units[lo:lo + 16])) == 1                       # one unit per run of 16
            steps = [int(tiles[t][5]) for (t, _) in body[lo:lo + 16]]
            assert steps == sorted(steps, reverse=True)
        steps = [int(tiles[t][5]) * int(tiles[t][2]) for (t, _) in tail]
        assert steps == sorted(steps, reverse=True)


@pytest.mark.parametrize("seed", range(20))
def test_plan_of_random_problems(B, seed):
    """Random sizes, branch sets (also ragged ones) and offsets: every (h, n) in exactly one tile, and every
    tile's progressions add up to exactly the multiset of keys the definition gives its rows."""
    rng = np.random.default_rng(50 + seed)
    Bsz, H, N, nb = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(1, 700)), int(rng.integers(1, 9))
    branches, offs = [], []
    for _ in range(nb):
        r = int(rng.integers(1, 8))
        branches.append((int(rng.integers(1, 2 * N + 1)), r))
        offs.append([int(rng.integers(0, r)) for _ in range(H)])
    offs = offs if seed % 2 else None
    p = B.plan_describe(Bsz, H, N, branches, offs)
    tiles, rows, segs, items = p["tiles"], p["rows"], p["segs"], p["items"]
    seen = np.zeros((H, N), dtype=np.int32)
    for (h, rb, nr, sb, ns, _) in tiles:
        assert 1 <= nr <= 256 and ns <= 32
        got = [tuple(int(x) for x in segs[s]) for s in range(sb, sb + ns)]
        for n in rows[rb:rb + nr]:
            seen[h, n] += 1
            counts, plain = _expected_multiset(N, h, int(n), branches, offs)
            _check_tile_list(N, got, counts, plain)
    assert np.all(seen == 1)
    real = items[items[:, 0] >= 0]
    assert len(items) % 8 == 0 and len(set(map(tuple, real.tolist()))) == len(real) == len(tiles) * Bsz


def _check_forward_plan(B, Bsz, H, N, branches, offs, sample=None):
    """The plan of the bf16 forward: every (h, n) is stored by exactly one slot, and for every slot (filler slots
    included: they are computed like the row they repeat) the progressions its 32-row block takes, with the block's
    multiplicities, add up to exactly the multiset of keys the definition gives the row."""
    p = B.plan_describe_forward(Bsz, H, N, branches, offs)
    tiles, rows, segs, wm, items = p["tiles"], p["rows"], p["segs"], p["block_mult"], p["items"]
    seen = np.zeros((H, N), dtype=np.int32)
    for (h, rb, nr, sb, ns, steps) in tiles:
        assert 1 <= nr <= 256 and ns <= 32
        assert steps == sum((int(c) + 63) // 64 for c in segs[sb:sb + ns, 2])
        tile_rows = rows[rb:rb + nr]
        assert tile_rows[0] >= 0 and tile_rows[-1] >= 0
        real = tile_rows[tile_rows >= 0]
        seen[h, real] += 1
        if ns:
            live = wm[sb:sb + ns, :(nr + 31) // 32]
            assert live.max(axis=0).min() >= 1 and live.max(axis=1).min() >= 1    # no idle block, no unused progression
            assert np.array_equal(segs[sb:sb + ns, 3], wm[sb:sb + ns].max(axis=1))
            assert np.all(wm[sb:sb + ns, (nr + 31) // 32:] == 0) or np.all(tile_rows >= 0)
        slots = range(nr) if sample is None else sample(nr)
        for slot in slots:
            n = int(tile_rows[slot])
            n = ~n if n < 0 else n
            w = slot // 32
            got = [(int(segs[s][0]), int(segs[s][1]), int(segs[s][2]), int(wm[s][w])) for s in range(sb, sb + ns) if wm[s][w] > 0]
            counts, _ = _expected_multiset(N, h, n, branches, offs)
            mine = np.zeros(N, dtype=np.int32)
            for (first, stride, count, mult) in got:
                assert count >= 1 and stride >= 1 and 0 <= first and first + stride * (count - 1) < N
                mine[first:first + stride * count:stride] += mult
            assert np.array_equal(mine, counts), (h, n, slot)
    assert np.all(seen == 1)
    real = items[items[:, 0] >= 0]
    assert len(items) % 8 == 0 and len(set(map(tuple, real.tolist()))) == len(real) == len(tiles) * Bsz
    return p


@pytest.mark.parametrize("Bsz,H,N,branches,offs", [
    (1, 1, 256, [(64, 2)], None),
    (16, 6, 256, [(64, 1), (128, 2), (256, 4)], None),
    (16, 12, 1024, [(256, 1), (512, 2), (1024, 4)], None),
    (1, 12, 4096, [(1024, 1), (2048, 2), (4096, 4)], None),
    (3, 4, 360, [(120, 3), (180, 2), (360, 5)], [[2, 0, 1, 2], [1, 1, 0, 0], [4, 3, 0, 1]]),
    (40, 2, 96, [(32, 4), (96, 1)], None),
    (2, 3, 50, [(16, 3), (7, 2), (64, 5)], None),
    (1, 2, 1025, [(1024, 1), (300, 7)], [[0, 0], [6, 2]]),
    (1, 2, 512, [(256, 2), (256, 2), (512, 1)], None),
    (2, 2, 700, [(100, 1), (350, 2), (700, 3), (50, 1)], None),
])
def test_forward_plan_covers_the_definition(B, Bsz, H, N, branches, offs):
    _check_forward_plan(B, Bsz, H, N, branches, offs)


@pytest.mark.parametrize("seed", range(20))
def test_forward_plan_of_random_problems(B, seed):
    rng = np.random.default_rng(150 + seed)
    Bsz, H, N, nb = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(1, 700)), int(rng.integers(1, 9))
    branches, offs = [], []
    for _ in range(nb):
        r = int(rng.integers(1, 8))
        branches.append((int(rng.integers(1, 2 * N + 1)), r))
        offs.append([int(rng.integers(0, r)) for _ in range(H)])
    _check_forward_plan(B, Bsz, H, N, branches, offs if seed % 2 else None)


def test_forward_plan_packs_the_row_groups_of_small_images(B):
    """512^2 image (N = 1024) with the workload's branch family: the rows of one window of the narrowest branch fall
    into groups of 128, 64 and 64 rows by which dilated branches also keep them; apart they are 12 part-filled
    tiles per head walking 4, 6 and 8 steps (72 in all), packed they are 4 full tiles of 8 steps (a group takes
    whole 32-row blocks of a tile, two to a wave).  At 1024^2 every
    group fills whole tiles and the plan is the plain one."""
    wl = lambda N: [(N // 4, 1), (N // 2, 2), (N, 4)]
    plain, packed = B.plan_describe(1, 12, 1024, wl(1024)), B.plan_describe_forward(1, 12, 1024, wl(1024))
    assert len(plain["tiles"]) == 12 * 12 and int(plain["tiles"][:, 5].sum()) == 12 * 72
    assert len(packed["tiles"]) == 12 * 4 and np.all(packed["tiles"][:, 2] == 256) and np.all(packed["tiles"][:, 5] == 8)
    assert np.all(packed["rows"] >= 0)
    # 256^2: groups of 32, 16 and 16 rows, one 32-row block each (filler slots up to the next block): 12 tiles of 1, 2
    # and 3 steps per head apart (24 steps), 2 tiles of six blocks and 4 steps packed
    plain, small = B.plan_describe(1, 6, 256, wl(256)), B.plan_describe_forward(1, 6, 256, wl(256))
    assert len(plain["tiles"]) == 6 * 12 and int(plain["tiles"][:, 5].sum()) == 6 * 24
    assert len(small["tiles"]) == 6 * 2 and np.all(small["tiles"][:, 2] == 192) and np.all(small["tiles"][:, 5] == 4)
    # heads 4 and 5 start at the offsets of heads 0 and 1 (h mod 1, 2, 4): their tiles point at the same rows and lists
    assert int((small["rows"] < 0).sum()) > 0 and int((small["rows"] >= 0).sum()) == 4 * 256
    assert np.array_equal(small["tiles"][8:, 1:], small["tiles"][:4, 1:]) and list(small["tiles"][8:, 0]) == [4, 4, 5, 5]
    plain, packed = B.plan_describe(1, 12, 4096, wl(4096)), B.plan_describe_forward(1, 12, 4096, wl(4096))
    for key in ("tiles", "rows", "segs", "items"):
        assert np.array_equal(plain[key], packed[key])
    assert np.all(packed["block_mult"] == packed["segs"][:, 3:4])


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
