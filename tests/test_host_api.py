"""Host-side checks that need no GPU: the library loads, exports what the
header declares, validates arguments and plans the Gram path."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2512_23353_amd import isopo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _host_layer(lengths, d_in, d_out, dtype=isopo.BF16):
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    return isopo.Layer(None, None, off, d_in=d_in, d_out=d_out, dtype=dtype, n_tokens=int(off[-1]))


def test_library_exports_every_declared_symbol():
    lib = isopo.load()
    header = open(os.path.join(ROOT, "include", "isopo.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(isopo_[a-z0-9_]+)\s*\(", header))
    assert declared == set(isopo.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert isopo.version() == "0.1"
    assert isopo.status_string(0) == "ok"
    assert "offset" in isopo.status_string(2)


def test_offsets_validation():
    lay = _host_layer([3, 4], 64, 64)
    assert isopo.gram_plan(lay)[0] in ("ghost", "materialised")
    for bad in ([1, 3, 7], [0, 5, 3, 7], [0, 3, 6]):
        lay = isopo.Layer(None, None, np.array(bad, dtype=np.int32), d_in=64, d_out=64, dtype=isopo.BF16, n_tokens=7)
        with pytest.raises(isopo.IsopoError) as e:
            isopo.gram_plan(lay)
        assert e.value.status == 2
    # zero-length sequences are legal
    assert isopo.gram_plan(_host_layer([0, 5, 0], 64, 64))[0] in ("ghost", "materialised")


def test_shape_and_dtype_validation():
    with pytest.raises(isopo.IsopoError) as e:
        isopo.gram_plan(_host_layer([4], 60, 64))          # d_in not a multiple of 8 for bf16
    assert e.value.status == 3
    assert isopo.gram_plan(_host_layer([4], 60, 64, isopo.F32))[0]   # fine for fp32 (multiple of 4)
    with pytest.raises(isopo.IsopoError) as e:
        isopo.gram_plan(_host_layer([4], 64, 64, dtype=7))
    assert e.value.status == 3
    with pytest.raises(isopo.IsopoError) as e:
        isopo.gram_plan(_host_layer([1] * (isopo.MAX_SEQ + 1), 64, 64))
    assert e.value.status == 3


def test_null_device_pointers_rejected_before_any_launch():
    lay = _host_layer([3, 4], 64, 64)
    lib = isopo.load()
    st = lib.isopo_layer_gram(lay.ref(), isopo.GRAM_AUTO, None, None, 0, 0, None)
    assert st == 1
    st = lib.isopo_weighted_grad(lay.ref(), None, None, 0.0, None, None)
    assert st == 1
    st = lib.isopo_transform(None, None, 4, 1, 0, 0.0, 0, None, None, None, 0, None)
    assert st == 1
    assert lib.isopo_layer_gram_plan(None, 0, None, None, None) == 1


def test_plan_workspace_sizes():
    lay = _host_layer([300, 200, 100], 512, 1024)
    path, full, mn = isopo.gram_plan(lay, "materialised")
    assert path == "materialised"
    stash = 3 * 1024 * 512 * 2
    assert full >= stash and mn < full and mn >= 3 * 256 * 512 * 2
    path, full, mn = isopo.gram_plan(lay, "ghost")
    assert path == "ghost" and full == mn and full >= 9 * 8 + 600 * 4
    lay32 = _host_layer([300, 200, 100], 512, 1024, isopo.F32)
    assert isopo.gram_plan(lay32, "materialised")[1] >= 2 * stash
    assert isopo.transform_workspace(128) == 0
    assert isopo.transform_workspace(256, 3) == 3 * (256 * 256 + 256) * 8


def test_cost_model_prefers_ghost_only_for_few_tokens():
    """Ghost costs ~N^2 (d_in + d_out) with a floor (one serial walk over the
    features), materialised ~2 N d_in d_out plus two passes over a stash of
    B d_in d_out elements: ghost must win for many short sequences on a wide
    layer and lose for a long microbatch, the modelled costs must order the
    same way as the AUTO choice, and once the microbatch is long enough for
    the materialised path it stays the choice."""
    small = _host_layer([8] * 32, 4096, 14336)
    big = _host_layer([2048] * 32, 4096, 14336)
    assert isopo.gram_plan(small)[0] == "ghost"
    assert isopo.gram_plan(big)[0] == "materialised"
    for lay in (small, big):
        tg, tm = isopo.gram_cost_model(lay)
        assert tg > 0 and tm > 0
        assert (isopo.gram_plan(lay)[0] == "ghost") == (tg < tm)
    # a narrow layer: the stash is small, so the materialised path wins as soon as the token-tile pairs
    # fill the chip and the ghost kernel no longer cuts its walk over the features into ranges
    assert isopo.gram_plan(_host_layer([64] * 4, 4096, 1024))[0] == "ghost"
    assert isopo.gram_plan(_host_layer([512] * 4, 4096, 1024))[0] == "materialised"
    choices, ghost_costs = [], []
    for t in (8, 64, 256, 512, 1024, 4096):
        lay = _host_layer([t] * 16, 5120, 27648)
        choices.append(isopo.gram_plan(lay)[0])
        ghost_costs.append(isopo.gram_cost_model(lay)[0])
    assert choices[0] == "ghost" and choices[-1] == "materialised"
    first_mat = choices.index("materialised")
    assert all(c == "materialised" for c in choices[first_mat:])
    assert all(a <= b for a, b in zip(ghost_costs, ghost_costs[1:]))


def test_stash_layout_is_a_host_function_of_dtype_and_shape():
    """Tile order for bf16 layers whose dimensions are multiples of 256 (the tile is the contraction plan's);
    row-major otherwise."""
    many = [64] * 48
    assert isopo.stash_layout(_host_layer(many, 768, 512)) == (isopo.STASH_TILE_ORDER, 256)
    assert isopo.stash_layout(_host_layer([70, 129, 33], 256, 512)) == (isopo.STASH_TILE_ORDER, 128)
    assert isopo.stash_layout(_host_layer(many, 4096, 14336)) == (isopo.STASH_TILE_ORDER, 256)
    assert isopo.stash_layout(_host_layer(many, 768, 520)) == (isopo.STASH_ROW_MAJOR, 0)
    assert isopo.stash_layout(_host_layer(many, 264, 512)) == (isopo.STASH_ROW_MAJOR, 0)
    assert isopo.stash_layout(_host_layer(many, 768, 512, dtype=isopo.F32)) == (isopo.STASH_ROW_MAJOR, 0)


def test_contraction_plan_whole_tiles_then_split_tail():
    """Unweighted contraction with more 256x256 tiles than compute units and a partial last round: the tiles
    of the full rounds stay whole, the rest is cut into token chunks that fill the round.  The kernel's
    decoding of (workgroup id -> tile, chunk), repeated here, must cover every whole tile once and every
    (chunk, tail tile) pair once."""
    for d_in, d_out, n_tok in ((4096, 14336, 70107), (5120, 27648, 412293), (4096, 4200, 2048)):
        lay = _host_layer([n_tok], d_in, d_out)
        pl = isopo.contraction_plan(lay.ref(), False)
        tiles, whole, w, ct = pl["tiles"], pl["whole_tiles"], pl["n_chunks"], pl["chunk_tokens"]
        assert tiles == -(-d_in // 256) * -(-d_out // 256)
        assert whole == tiles // 256 * 256 and w > 1
        rest = tiles - whole
        assert rest * w <= 256 and ct % 32 == 0 and (w - 1) * ct < n_tok <= w * ct
        assert pl["workgroups"] % 8 == 0
        seen_whole, seen_split = [], []
        for b in range(pl["workgroups"]):
            x, e = b & 7, b >> 3
            wq = whole >> 3
            if e < wq:
                seen_whole.append(x * wq + e)
                continue
            S = rest * w
            first, last = x * S // 8, (x + 1) * S // 8
            idx = first + (e - wq)
            if idx < last:
                seen_split.append((idx // rest, whole + idx % rest))
        assert sorted(seen_whole) == list(range(whole))
        assert sorted(seen_split) == [(c, t) for c in range(w) for t in range(whole, tiles)]
    # a multiple of 256 tiles, or fewer than 256: nothing to fill
    assert isopo.contraction_plan(_host_layer([70107], 4096, 4096).ref(), False)["whole_tiles"] == 0
    assert isopo.contraction_plan(_host_layer([131072], 1536, 8960).ref(), False)["whole_tiles"] == 0
    # per-sequence mode never splits tokens
    assert isopo.contraction_plan(_host_layer([70107], 4096, 14336).ref(), True)["whole_tiles"] == 0


def test_contraction_plan_ranges_partition_the_work():
    """Launch plan of the per-sequence contraction.  Tile counts that are a
    multiple of eight keep the tile-eighths mapping (no range list); otherwise
    the eight XCD ranges must tile [0, n_seq * tiles) exactly, in order, and
    carry equal work up to one pair."""
    # config-3 shapes: 256, 64, 896 tiles -> eighths
    for d_in, d_out in ((4096, 4096), (4096, 1024), (4096, 14336)):
        plan = isopo.contraction_plan(_host_layer([2048] * 32, d_in, d_out).ref(), True)
        assert plan["tile"] == 256 and plan["tiles"] % 8 == 0
        assert plan["xcd_start"] == [0] * 9
        assert plan["workgroups"] == 32 * plan["tiles"]
    rng = np.random.default_rng(5)
    cases = [([2048] * 64, 1536, 1536), ([2048] * 64, 1536, 256), ([2048] * 64, 1536, 8960),
             (list(rng.integers(256, 1025, 16)), 1536, 1536), (list(rng.integers(1, 3000, 37)), 1536, 8960),
             ([0, 5, 0, 700, 0], 1536, 256), ([100, 0, 5000], 1536, 256)]
    checked = 0
    for lengths, d_in, d_out in cases:
        plan = isopo.contraction_plan(_host_layer(lengths, d_in, d_out).ref(), True)
        tiles, st = plan["tiles"], plan["xcd_start"]
        if tiles % 8 == 0:                      # few sequences on a narrow layer: 128-wide tiles, 24 of them
            assert plan["tile"] == 128 and st == [0] * 9
            continue
        checked += 1
        assert st[0] == 0 and st[8] == len(lengths) * tiles
        assert all(a <= b for a, b in zip(st, st[1:]))
        assert plan["workgroups"] == 8 * max(b - a for a, b in zip(st, st[1:]))
        # equal work: tokens + 192 per pair, no XCD more than one pair's work above the mean
        w = np.asarray(lengths) + 192
        work = [int(np.sum(w[np.arange(st[x], st[x + 1]) // tiles])) for x in range(8)]
        assert sum(work) == int(np.sum(w)) * tiles
        assert max(work) <= sum(work) / 8 + int(w.max()), (lengths[:4], d_in, d_out, work)
    assert checked >= 5


def test_contraction_plan_token_split():
    """Unweighted mode.  Enough tiles: no split.  Few tiles and many tokens: a
    split whose (chunk, tile) pairs fit the 32 CUs of an XCD in whole rounds,
    chunks a multiple of the 32-token block, covering all tokens; a split is
    never chosen when its atomic adds would cost more than the idle CUs."""
    # 4096x4096 on 70k tokens: 256 tiles fill the chip
    plan = isopo.contraction_plan(_host_layer([70107], 4096, 4096).ref(), False)
    assert (plan["n_chunks"], plan["chunk_tokens"], plan["xcd_start"]) == (1, 70107, [0] * 9)
    assert plan["workgroups"] == plan["tiles"] == 256
    # config-4 q: 36 tiles, 131072 tokens -> 7 chunks = 252 pairs, 31 or 32 per XCD
    plan = isopo.contraction_plan(_host_layer([2048] * 64, 1536, 1536).ref(), False)
    assert plan["tile"] == 256 and plan["tiles"] == 36 and plan["n_chunks"] == 7
    assert plan["chunk_tokens"] % 32 == 0 and plan["chunk_tokens"] * 7 >= 131072 > plan["chunk_tokens"] * 6
    st = plan["xcd_start"]
    assert st[0] == 0 and st[8] == 252 and all(31 <= b - a <= 32 for a, b in zip(st, st[1:]))
    assert plan["workgroups"] == 256
    # 210 tiles on 10k tokens: splitting would add 13.8M atomic adds per chunk for little gain
    plan = isopo.contraction_plan(_host_layer([10365], 1536, 8960).ref(), False)
    assert plan["n_chunks"] == 1
    # narrow layer, short microbatch: the small tile, and some split
    plan = isopo.contraction_plan(_host_layer([3000, 1400, 1, 4200, 333, 4100], 256, 384).ref(), False)
    assert plan["tile"] == 128 and plan["workgroups_per_cu"] == 2 and plan["n_chunks"] > 1
    assert plan["chunk_tokens"] % 32 == 0 and plan["chunk_tokens"] * plan["n_chunks"] >= 13034
    assert plan["xcd_start"][8] == plan["n_chunks"] * plan["tiles"]
    # nothing to do
    plan = isopo.contraction_plan(_host_layer([0, 0], 256, 256).ref(), False)
    assert plan["n_chunks"] == 1
    # fp32 inputs do not use this kernel
    with pytest.raises(isopo.IsopoError) as e:
        isopo.contraction_plan(_host_layer([64], 64, 64, dtype=isopo.F32).ref(), True)
    assert e.value.status == 3


def test_contraction_plan_invariants_on_random_shapes():
    """Four hundred random layers (widths multiples of 8 from 8 to 9000, 1 to 300 sequences of 0 to 5000
    tokens) through the launch plan in both modes: whatever the plan, it must describe a launch that
    covers every (item, tile) pair once and every token once."""
    rng = np.random.default_rng(2024)
    for case in range(400):
        d_in = int(rng.choice([8, 64, 72, 256, 384, 1024, 1536, 4096, 8960])) if case % 3 else 8 * int(rng.integers(1, 1125))
        d_out = int(rng.choice([8, 136, 256, 512, 1536, 4096, 14336])) if case % 2 else 8 * int(rng.integers(1, 1125))
        n_seq = int(rng.integers(1, 300)) if case % 5 else int(rng.integers(1, 9))
        lengths = rng.integers(0, int(rng.choice([3, 40, 600, 5000])), n_seq)
        if case % 7 == 0:
            lengths[:] = 0
        n_tok = int(lengths.sum())
        lay = _host_layer(list(lengths), d_in, d_out)
        for per_seq in (True, False):
            pl = isopo.contraction_plan(lay.ref(), per_seq)
            what = (case, d_in, d_out, n_seq, n_tok, per_seq, pl)
            T = pl["tile"]
            assert T in (128, 256), what
            tiles = -(-d_in // T) * -(-d_out // T)
            assert pl["tiles"] == tiles and pl["workgroups_per_cu"] in (1, 2), what
            st, w, ct, whole = pl["xcd_start"], pl["n_chunks"], pl["chunk_tokens"], pl["whole_tiles"]
            assert w >= 1 and 0 <= whole <= tiles, what
            if per_seq:
                assert w == 1 and whole == 0, what
                items = n_seq
            else:
                items = w
                if w > 1:
                    assert ct % 32 == 0 and (w - 1) * ct < n_tok <= w * ct, what
                else:
                    assert ct >= n_tok, what
            if whole:
                # whole tiles in rounds of 256, the rest cut into chunks that fit one more round
                assert not per_seq and whole % 256 == 0 and whole < tiles and w > 1 and (tiles - whole) * w <= 256, what
                assert st == [0] * 9, what
                continue
            if st[8] > 0:
                assert st[0] == 0 and st[8] == items * tiles and all(a <= b for a, b in zip(st, st[1:])), what
                assert pl["workgroups"] == 8 * max(b - a for a, b in zip(st, st[1:])), what
            else:
                assert st == [0] * 9, what
                if per_seq or w > 1:
                    assert tiles % 8 == 0 and pl["workgroups"] == items * tiles, what      # eighths of every item's tiles
                else:
                    assert pl["workgroups"] == tiles, what


def test_bench_refuses_more_than_one_gpu():
    """The layer step has no cross-GPU part: bench.py --gpus N > 1 exits with a
    message instead of printing a number (and touches no GPU on the way)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")


def test_bench_reads_the_committed_traffic_summary():
    # roofline.traffic comes from the counter summary under profiles/: the line bench.py parses is there and
    # equals the sum of the read and written bytes the same file states
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    traffic = bench.read_traffic("seq_grad_config3")
    assert traffic is not None and traffic > 0
    text = open(os.path.join(root, "profiles", "seq_grad_config3_hbm_traffic.txt")).read()
    read = float(re.search(r"FETCH_SIZE mean .*-> ([0-9.e]+) B read", text).group(1))
    written = float(re.search(r"WRITE_SIZE mean .*-> ([0-9.e]+) B written", text).group(1))
    assert abs(traffic - (read + written)) <= 0.005 * traffic
    assert bench.read_traffic("no_such_kernel") is None
