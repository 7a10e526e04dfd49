"""Host logic of the segment / tile tables (no GPU): what the kernels would be told to do.

The oracle side is only the definition of the merged order: groups in communication order,
layers inside a group from the highest down (Algorithm 2 pushes layers as their backward pass
ends), offsets = running element counts without padding (Condition 3)."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import planner as op
from paper_1811_11141_amd import binding as mg
from paper_1811_11141_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def expected_segments(p, merged, pad=1):
    """[(layer0, n, plan offset, group)] in merged order, from the oracle's grouping; with
    pad > 1 every layer starts on a multiple of pad elements."""
    rows, off = [], 0
    for k, grp in enumerate(op.groups_from_merged(len(p), merged)):
        for l in grp:
            rows.append((l - 1, int(p[l - 1]), off, k))
            off += -(-int(p[l - 1]) // pad) * pad
    return rows


def check_layout(p, merged, tile, small, long_tiles=-1, pad=0):
    L = len(p)
    pl = mg.mgwfbp_plan_explicit(p, np.ones(L), 0.0, 0.5, 1e-6, 2, merged)
    t_iter = pl.info()["t_iter_ms"]
    pl.set_option(mg.OPT_TILE_ELEMS, tile)
    pl.set_option(mg.OPT_SMALL_ELEMS, small)
    pl.set_option(mg.OPT_LONG_TILES, long_tiles)
    pl.set_option(mg.OPT_PAD_ELEMS, pad)
    pq = max(pad, 1)
    plen = lambda n: -(-n // pq) * pq
    lay = pl.layout()
    segs, tiles = lay["segments"], lay["tiles"]
    exp = expected_segments(p, merged, pq)
    assert [tuple(int(x) for x in r) for r in segs] == exp
    P = sum(plen(int(x)) for x in p)                      # the merged order, padding included
    inf = pl.info()
    assert inf["t_iter_ms"] == t_iter                     # the cost model counts 4 * sum p bytes
    assert int(inf["group_elems"].sum()) == P
    for lyr, n, off, grp in exp:
        assert int(inf["group_of_layer"][lyr]) == grp
    gstart = {}
    for lyr, n, off, grp in exp:
        gstart.setdefault(grp, off)
        assert int(inf["offset_in_group"][lyr]) == off - gstart[grp]
        assert pad == 0 or off % pad == 0
    small_eff = min(small, tile)
    lists = sorted({int(x) for x in tiles[:, 4]})
    assert lists[:2] == [0, 1] and (2 in lists) == (long_tiles not in (-1, 0) and tile == 4096) and 4 in lists
    for which in lists:       # per-group lists, whole-plan list, double-length list, arrival-ordered list
        cover = np.zeros(P, dtype=np.uint8)
        sel = tiles[tiles[:, 4] == which]
        assert len(sel) > 0
        last_group, seen_full_in_group = -1, False
        for first, nseg, start, n, _, tlen, tpad in (tuple(int(x) for x in r) for r in sel):
            if which in (2, 3):
                assert tlen == (8192 if long_tiles == 1 else long_tiles) and 1 <= n <= tlen
            elif which == 4:
                # the arrival-ordered list has tile lengths of its own, whatever tile_elems says: 512 for
                # small groups, else 1024 while the plan is at most 2 * 14 * 256 tiles of 4096 elements
                gsz = sum(plen(e[1]) for e in exp if e[3] == exp[first][3])
                assert tlen == (512 if gsz <= 64 * 1024 else (1024 if -(-P // 4096) <= 7168 else 4096))
                assert 1 <= n <= max(tlen, min(tile, 1024), small_eff)
            else:
                assert 1 <= n <= tile, "no tile exceeds tile_elems (the LDS staging size)"
                # a group's own list may use shorter tiles than the whole-plan list, never longer
                assert tlen in (tile, tile // 2, tile // 4) and tlen >= 1024 and (which == 0 or tlen == tile)
            assert 1 <= nseg <= 256
            if nseg == 1:
                lyr, sn, soff, grp = exp[first]
                assert start + n <= sn, "direct tile stays inside its segment"
                assert start % tlen == 0
                assert n == tlen or start + n == sn, "only the last piece of a segment is ragged"
                assert tpad == (plen(sn) - sn if start + n == sn else 0), "the last piece owns the layer's padding"
                lo = soff + start
                is_full = n == tlen              # before the padding it owns is counted in
                n += tpad
            else:
                members = exp[first:first + nseg]
                assert all(m[1] < small_eff for m in members), "gather tiles hold short layers only"
                assert len({m[3] for m in members}) == 1, "a gather tile never crosses a group"
                assert start == members[0][2] and n == sum(plen(m[1]) for m in members) and tpad == 0
                assert n <= max(min(tile, 1024), small_eff)
                grp = members[0][3]
                lo = start
                is_full = False
            cover[lo:lo + n] += 1
            if which in (0, 4):
                # group after group; inside a group the slow tiles (gather, ragged) come first
                assert grp >= last_group
                if grp != last_group:
                    last_group, seen_full_in_group = grp, False
                full = is_full
                assert not (seen_full_in_group and not full), "slow tile after a full tile"
                seen_full_in_group = seen_full_in_group or full
        assert cover.min() == 1 and cover.max() == 1, "every element in exactly one tile"
        if which == 0:
            # the shorter tiles are there to give a short launch enough workgroups
            for k, grp in enumerate(op.groups_from_merged(len(p), merged)):
                ge = sum(plen(int(p[l - 1])) for l in grp)
                tl_k = {int(r[5]) for r in sel if exp[int(r[0])][3] == k}
                assert len(tl_k) == 1
                t_k = tl_k.pop()
                assert t_k == tile or -(-ge // (2 * t_k)) < 2048, "halved only while the launch is short"
    pl.destroy()


@pytest.mark.parametrize("tile,small", [(1024, 0), (1024, 512), (4096, 512), (4096, 8192), (8192, 1), (2048, 2048)])
def test_layout_tiny_nets(tile, small):
    for seed in range(6):
        w = wl.tiny_workload(seed, L=10)
        rng = np.random.default_rng(seed)
        merged = [l for l in range(2, w.L + 1) if rng.random() < 0.5]
        check_layout(w.p, merged, tile, small)


@settings(max_examples=60, deadline=None, derandomize=True)
@given(st.lists(st.integers(1, 20000), min_size=1, max_size=30), st.data(),
       st.sampled_from([1024, 2048, 4096, 8192]), st.sampled_from([0, 1, 64, 512, 1024, 4096, 8192]))
def test_layout_random(p, data, tile, small):
    L = len(p)
    merged = [l for l in range(2, L + 1) if data.draw(st.booleans())]
    check_layout(np.array(p, dtype=np.uint64), merged, tile, small)


@pytest.mark.parametrize("seed", range(4))
def test_layout_double_length_list(seed):
    w = wl.tiny_workload(seed, L=12)
    rng = np.random.default_rng(seed)
    merged = [l for l in range(2, w.L + 1) if rng.random() < 0.5]
    check_layout(w.p, merged, 4096, 512, long_tiles=1)
    check_layout(w.p, merged, 4096, 512, long_tiles=0)
    for tlen in (5120, 6144, 7168, 8192):
        check_layout(w.p, merged, 4096, 512, long_tiles=tlen)
    check_layout(w.p, merged, 2048, 512, long_tiles=1)     # only built for 4096-element tiles


def test_longer_tile_list_is_chosen_by_launch_size():
    """The whole-plan reduce pass gets the tile length that fills the chip's batches of workgroups
    best.  Expected choices for single tensors of k thousand 4096-element tiles, from the rule
    (16 workgroups per compute unit, 14 with 16 workers or 8192-element tiles, 256 units; a last
    batch under 65 % full costs a 65 % one; a launch that fits the chip at once is best with
    11-13 workgroups per unit; a longer tile must gain 2 %) -- they are also the
    lengths that measured best or within 1 % of the best on MI355X."""
    def chosen(k_tiles, n_workers):
        n = int(k_tiles * 1000) * 4096 + 1234 * 4
        pl = mg.mgwfbp_plan([n], [1.0], 0.0, 0.5, 1e-6, n_workers, mg.MODE_WFBP)
        t = pl.layout()["tiles"]
        pl.destroy()
        default = t[t[:, 4] == 2]
        return int(default[0, 5]) if len(default) else 4096
    expect8 = {3: 4096, 4: 5120, 5: 7168, 6.4: 8192, 7: 4096, 8: 4096, 9: 5120, 10: 5120, 12: 4096, 18: 6144, 24: 4096}
    expect16 = {3: 4096, 4: 5120, 5: 7168, 6.4: 4096, 8: 5120, 9: 6144, 10: 4096, 12: 5120, 15: 6144, 18: 7168, 24: 4096}
    assert {k: chosen(k, 8) for k in expect8} == expect8
    assert {k: chosen(k, 16) for k in expect16} == expect16
    for name, tlen in (("resnet50", 8192), ("googlenet", 4096), ("alexnet", 4096)):
        w = wl.cnn_workload(name)
        pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
        tiles = pl.layout()["tiles"]
        default = tiles[tiles[:, 4] == 2]
        assert (int(default[0, 5]) if len(default) else 4096) == tlen, name
        for which in (2, 3):
            sel = tiles[tiles[:, 4] == which]
            if len(sel):
                assert int(sel[:, 3].sum()) == w.P and len(sel) >= 2048
        pl.destroy()


@pytest.mark.parametrize("tile,small", [(1024, 0), (1024, 512), (4096, 512), (4096, 1026), (2048, 2048)])
def test_layout_padded(tile, small):
    """MGWFBP_OPT_PAD_ELEMS = 4, 8, 16, 32: every layer starts on a multiple of that many
    elements, the tiles cover the padded merged order exactly once, the predicted times do not move."""
    for seed in range(6):
        rng = np.random.default_rng(50 + seed)
        L = int(rng.integers(1, 30))
        p = np.array([int(rng.integers(1, 3000)) if rng.random() < 0.7 else int(rng.integers(3000, 40000))
                      for _ in range(L)], dtype=np.uint64)
        merged = [l for l in range(2, L + 1) if rng.random() < 0.6]
        check_layout(p, merged, tile, small, pad=4)
        check_layout(p, merged, tile, small, long_tiles=1, pad=4)
        check_layout(p, merged, tile, small, pad=(8, 16, 32)[seed % 3])


def test_layout_many_tiny_layers_split_gather_tiles():
    """300 layers of 3 elements in one group: more than 256 segments cannot share one tile."""
    p = np.full(300, 3, dtype=np.uint64)
    check_layout(p, list(range(2, 301)), 4096, 512)


def test_layout_cnn_sets_default_options():
    for name, n_tiles_min in (("resnet50", 6000), ("vgg16", 33000)):
        w = wl.cnn_workload(name)
        pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
        lay = pl.layout()
        whole = lay["tiles"][lay["tiles"][:, 4] == 1]
        assert len(whole) >= n_tiles_min
        assert int(whole[:, 3].sum()) == w.P
        full = whole[(whole[:, 1] == 1) & (whole[:, 3] == 4096)]
        assert int(full[:, 3].sum()) > 0.97 * w.P          # the bulk runs the fast path
        merged = pl.merged_layers()
        assert [tuple(int(x) for x in r) for r in lay["segments"]] == expected_segments(w.p, merged)
        pl.destroy()


def test_layout_thresholds_exactly():
    """The three size thresholds of the table builder at their edges."""
    def lists_of(p, merged, opts=()):
        pl = mg.mgwfbp_plan_explicit(np.array(p, dtype=np.uint64), np.ones(len(p)), 0.0, 0.5, 1e-6, 4, merged)
        for k, v in opts:
            pl.set_option(k, v)
        t = pl.layout()["tiles"]
        pl.destroy()
        return t

    # a gather tile holds at most 1024 elements: 511 + 511 fit, the next 8 do not
    small512 = [(mg.OPT_SMALL_ELEMS, 512)]
    t = lists_of([8, 511, 511], [2, 3], small512)
    own = t[t[:, 4] == 0]
    assert [(int(r[1]), int(r[3])) for r in own] == [(2, 1022), (1, 8)]
    t = lists_of([2, 511, 511], [2, 3], small512)
    assert [(int(r[1]), int(r[3])) for r in t[t[:, 4] == 0]] == [(3, 1024)]
    # by default only layers under 64 elements share gather tiles
    # (communication order: 63 | 64 | 63 + 8; a lone short layer is a direct tile)
    t = lists_of([8, 63, 64, 63], [2, 3, 4])
    assert [(int(r[1]), int(r[3])) for r in t[t[:, 4] == 0]] == [(1, 63), (1, 64), (2, 71)]
    # a group's own list keeps 4096-element tiles from 2048 tiles on, and halves below
    for n_tiles, tlen in ((2048, 4096), (2047, 2048), (1024, 2048), (1023, 1024)):
        t = lists_of([n_tiles * 4096], [])
        own = t[t[:, 4] == 0]
        assert {int(x) for x in own[:, 5]} == {tlen}, (n_tiles, tlen)


def test_layout_lone_short_layer_of_exactly_one_tile_length():
    """Found by a long property run: two short layers that do not fit one gather tile become lone
    direct tiles; the one that is exactly one tile long counts as a full tile (listed after the
    ragged one)."""
    p = np.array([1] * 11 + [2049, 2048], dtype=np.uint64)
    check_layout(p, [13], 8192, 4096)


def _launch_rules(tmp_path, *args):
    import subprocess
    exe = str(tmp_path / "launch_rules")
    if not os.path.exists(exe):
        csrc = os.path.join(ROOT, "paper_1811_11141_amd", "csrc")
        cmd = ["g++", "-std=c++17", "-O1", "-I", csrc, "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__",
               os.path.join(ROOT, "tests", "capi", "launch_rules.cpp"), os.path.join(csrc, "tables.cpp"), "-o", exe]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
    out = subprocess.run([exe, *[str(a) for a in args]], capture_output=True, text=True, check=True).stdout
    return {int(a): int(b) for a, b in (ln.split() for ln in out.splitlines())}


def test_update_kernel_occupancy_rule(tmp_path):
    """Workgroups per compute unit of the update kernel, chosen per launch.  The rule may only
    answer with the LDS sizes measured to give 11, 10, 9, 8 workgroups per unit; it leaves short
    launches, other LDS sizes and worker counts without a fast path alone; and on the launch sizes
    of the MI355X sweeps it caps exactly where the uncapped launch sat in a dip (N = 8: 4002, 4502,
    5002, 5502, 7502, 8002, 11002 workgroups lost 4.5-7 % uncapped) and nowhere it sat on a peak
    (3002, 6002, 6502, 9002, 10002)."""
    KB160 = 160 * 1024
    sizes = [100, 2047, 3002, 3502, 4002, 4502, 5002, 5502, 6002, 6502, 7002, 7502, 8002, 9002, 10002,
             11002, 14002, 20002, 34002, 10**6]
    for n in (1, 2, 4, 8, 16):
        r = _launch_rules(tmp_path, "update", n, 256, KB160, -1, *sizes)
        assert set(r.values()) <= {0, 11000, 12500, 14000, 16000}
        assert r[100] == 0 and r[2047] == 0 and r[10**6] == 0
    r8 = _launch_rules(tmp_path, "update", 8, 256, KB160, -1, *sizes)
    assert all(r8[w] != 0 for w in (4002, 4502, 5002, 5502, 7502, 8002, 11002))
    assert all(r8[w] == 0 for w in (3002, 3502, 6002, 6502, 9002, 10002, 14002, 20002, 34002))
    r16 = _launch_rules(tmp_path, "update", 16, 256, KB160, -1, *sizes)
    assert all(r16[w] != 0 for w in (3502, 4002, 4502, 5002, 6502, 7002, 7502, 8002))
    assert all(r16[w] == 0 for w in (3002, 6002, 9002, 20002, 34002))
    # left alone: run-time worker counts, another LDS size, the rule switched off
    assert set(_launch_rules(tmp_path, "update", 3, 256, KB160, -1, *sizes).values()) == {0}
    assert set(_launch_rules(tmp_path, "update", 8, 256, 64 * 1024, -1, *sizes).values()) == {0}
    assert set(_launch_rules(tmp_path, "update", 8, 256, KB160, 0, *sizes).values()) == {0}
    # forced: one fixed size whatever the launch
    for per_cu, lds in ((11, 11000), (10, 12500), (9, 14000), (8, 16000)):
        assert set(_launch_rules(tmp_path, "update", 8, 256, KB160, per_cu, *sizes).values()) == {lds}
    # a chip with half the compute units reaches the same fill with half the workgroups
    half = _launch_rules(tmp_path, "update", 8, 128, KB160, -1, 1023, 2001, 2251, 2501, 3001, 3251)
    assert half[2501] == r8[5002] and half[3001] == r8[6002] and half[3251] == r8[6502]
    assert half[1023] == 0 and half[2001] == r8[4002]       # "short" is 8 workgroups per compute unit
