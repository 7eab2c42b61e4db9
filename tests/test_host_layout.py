"""Group / offset table and the tile tables of the library against the oracle's layout (bit-exact),
on the CPU: the kernels' owner lookup is replayed in Python from the very tables they read."""
import numpy as np
import pytest

import paper_1912_09268_amd as M
import workloads as W
from oracle import plan as OP


def _oracle_owner_map(n_elems, merged, group_base, arena_elems):
    """arena element -> (tensor, element inside tensor), -1 where the arena is padding."""
    tg, off, ge = OP.merge_layout(n_elems, merged)
    owner = np.full(arena_elems, -1, np.int64)
    inner = np.full(arena_elems, -1, np.int64)
    for i, n in enumerate(n_elems):
        s = int(group_base[tg[i]]) + off[i]
        owner[s:s + n] = i
        inner[s:s + n] = np.arange(n)
    return owner, inner


def _replay_kernel_lookup(tab, tile_elems, arena_elems, vec=4, block=256):
    """What the kernels do with the tables: fast path for single-tensor full tiles, else a prefix sum
    over segment lengths followed by a per-vector search, element-wise for straddling vectors."""
    owner = np.full(arena_elems, -1, np.int64)
    inner = np.full(arena_elems, -1, np.int64)
    for t, h in enumerate(tab["tiles"]):
        base = t * tile_elems
        valid, nseg, seg0 = int(h["valid"]), int(h["nseg"]), int(h["seg0"])
        if valid == tile_elems and nseg == 1:
            owner[base:base + tile_elems] = int(h["layer0"])
            inner[base:base + tile_elems] = -int(h["first_start"]) + np.arange(tile_elems)
            continue
        # tile-local segment starts: entry 1 is first_end, then running sum of interior lengths
        start = [None, int(h["first_end"])] if nseg > 1 else [None]
        for j in range(2, nseg):
            start.append(start[-1] + int(tab["seg_n"][seg0 + j - 1]))
        layer = [int(tab["seg_layer"][seg0 + j]) for j in range(nseg)]
        assert layer[0] == int(h["layer0"])

        def src(j, q):
            return q - int(h["first_start"]) if j == 0 else q - start[j]

        for p in range(0, valid, vec):
            lo, hi = 0, nseg - 1
            while lo < hi:
                mid = (lo + hi + 1) >> 1
                if start[mid] <= p:
                    lo = mid
                else:
                    hi = mid - 1
            j = lo
            end_j = start[j + 1] if j + 1 < nseg else valid
            if p + vec <= end_j:
                owner[base + p:base + p + vec] = layer[j]
                inner[base + p:base + p + vec] = src(j, p) + np.arange(vec)
            else:
                for q in range(p, min(p + vec, valid)):
                    while j + 1 < nseg and q >= start[j + 1]:
                        j += 1
                    owner[base + q] = layer[j]
                    inner[base + q] = src(j, q)
    return owner, inner


def _check_profile(n_elems, merged, P=4, dtype=M.F32):
    n_elems = [int(x) for x in n_elems]
    merged = [int(x) for x in merged]
    ctx = M.Context(n_elems, merged, P, dtype, host_only=True)
    off, grp, base, ge = ctx.layout()
    tg_o, off_o, ge_o = OP.merge_layout(n_elems, merged)
    assert grp.tolist() == tg_o
    assert off.tolist() == off_o
    assert ge.tolist() == ge_o
    assert ctx.n_groups == len(ge_o) and ctx.L == len(n_elems)
    # bases: tile aligned, slices disjoint and in arrival order
    tile = ctx.tile_elems
    assert all(int(b) % tile == 0 for b in base)
    for k in range(ctx.n_groups - 1):
        assert int(base[k]) + int(ge[k]) <= int(base[k + 1])
    if ctx.n_groups:
        assert int(base[-1]) + int(ge[-1]) <= ctx.arena_elems
    assert ctx.arena_elems == ctx.n_tiles * tile
    tab = ctx.tables()
    assert tab["group_tile"][0] == 0 and tab["group_tile"][-1] == ctx.n_tiles
    assert int(tab["seg_off"][-1]) == ctx.arena_elems
    ctx.close()
    return tab, base, tile, ctx.arena_elems


def test_layout_worked_example():
    ctx = M.Context([10, 20, 30, 40, 50, 60], [0, 1, 0, 0, 1, 1], P=2, host_only=True)
    off, grp, base, ge = ctx.layout()
    assert grp.tolist() == [2, 2, 1, 0, 0, 0]
    assert off.tolist() == [20, 0, 0, 110, 60, 0]
    assert ge.tolist() == [150, 30, 30]
    ctx.close()


@pytest.mark.parametrize("seed", range(12))
def test_tables_replay_matches_oracle_on_random_small_models(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(1, 120))
    hi = [40, 600, 5000, 30000][seed % 4]
    n = [int(x) for x in np.maximum(1, np.rint(np.exp(rng.uniform(0, np.log(hi), size=L))))]
    if L > 3:
        n[int(rng.integers(0, L))] = 0
        n[int(rng.integers(0, L))] = 0
    merged = [0] + [int(x) for x in (rng.random(L - 1) < [0.9, 0.5, 0.2][seed % 3])]
    tab, base, tile, arena = _check_profile(n, merged)
    got = _replay_kernel_lookup(tab, tile, arena)
    ref = _oracle_owner_map(n, merged, base, arena)
    assert np.array_equal(got[0], ref[0])
    assert np.array_equal(got[1], ref[1])


def test_tables_many_one_element_tensors():
    # more segments in a tile than the kernels stage in LDS (two per lane): exercises long prefix sums
    n = [1] * 3000 + [5, 1, 1, 7] * 50
    merged = [0] + [1] * (len(n) - 1)
    tab, base, tile, arena = _check_profile(n, merged)
    assert int(tab["tiles"]["nseg"].max()) == tile          # a tile of one-element tensors: more than any lane count x 2
    got = _replay_kernel_lookup(tab, tile, arena)
    ref = _oracle_owner_map(n, merged, base, arena)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


@pytest.mark.parametrize("name", ["toy_mlp", "resnet50", "tiny_layers"])
def test_tables_replay_on_profiles(name):
    p = W.make_profile(name)
    merged, _ = M.plan(p.size_bytes, p.t_backward, p.a, p.b)
    tab, base, tile, arena = _check_profile(p.n_elems, merged, p.P)
    if name == "resnet50":      # replaying 25 M elements in Python is slow: check the tile headers instead
        h = tab["tiles"]
        full = (h["valid"] == tile) & (h["nseg"] == 1)
        assert full.mean() > 0.95
        return
    got = _replay_kernel_lookup(tab, tile, arena)
    ref = _oracle_owner_map([int(x) for x in p.n_elems], merged.tolist(), base, arena)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


@pytest.mark.parametrize("name", ["vgg16", "transformer"])
def test_layout_of_large_profiles(name):
    p = W.make_profile(name)
    merged, _ = M.plan(p.size_bytes, p.t_backward, p.a, p.b)
    tab, base, tile, arena = _check_profile(p.n_elems, merged, p.P, M.BF16 if p.grad_dtype == "bf16" else M.F32)
    h = tab["tiles"]
    # every tile's first segment really contains the tile start
    t_idx = np.arange(h.shape[0], dtype=np.int64)
    seg_start = tab["seg_off"][h["seg0"]].astype(np.int64)
    assert np.array_equal(seg_start - t_idx * tile, h["first_start"])
    assert (h["first_start"] <= 0).all() and (h["valid"] >= 1).all() and (h["valid"] <= tile).all()
    assert np.array_equal(tab["seg_layer"][h["seg0"]], h["layer0"])


def test_empty_model_and_all_empty_tensors():
    ctx = M.Context([], [], P=1, host_only=True)
    assert (ctx.L, ctx.n_groups, ctx.arena_elems, ctx.n_tiles) == (0, 0, 0, 0)
    ctx.close()
    ctx = M.Context([0, 0, 5], [0, 1, 0], P=1, host_only=True)
    off, grp, base, ge = ctx.layout()
    assert ge.tolist() == [5, 0] and grp.tolist() == [1, 1, 0] and off.tolist() == [0, 0, 0]
    assert ctx.n_tiles == 1
    ctx.close()
