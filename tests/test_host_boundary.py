"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, validates descriptors, and its chunk store matches the oracle's model."""
import os
import re

import numpy as np
import pytest

import oracle.hcache_oracle as oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hc():
    import paper_2410_05004_amd as hc
    return hc


def header_symbols():
    text = open(os.path.join(ROOT, "include", "hcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(hc):
    syms = header_symbols()
    assert len(syms) >= 18
    for s in syms:
        assert hasattr(hc.lib, s), f"{s} declared in hcache.h but not exported"
    from paper_2410_05004_amd.binding import EXPORTED
    assert sorted(EXPORTED) == syms, "binding and header disagree on the entry points"


def test_version_and_error_string(hc):
    assert hc.version().startswith("hcache-mi355x")
    assert hc.lib.hc_last_error() is not None


def good_desc(hc, **over):
    kw = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, block_size=16,
              max_position=128, rope_style=0, rope_theta=10000.0, rms_eps=1e-5, norm_kind=0)
    kw.update(over)
    return hc.ModelDesc(*[kw[k] for k in ("n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                           "head_dim", "block_size", "max_position", "rope_style",
                                           "rope_theta", "rms_eps", "norm_kind")])


def test_desc_validation(hc):
    hc.validate_desc(good_desc(hc))
    hc.validate_desc(good_desc(hc, rope_style=2, norm_kind=1))
    bad = [dict(n_layers=0), dict(d_model=100), dict(head_dim=48), dict(n_q_heads=6, n_kv_heads=4),
           dict(block_size=12), dict(max_position=0), dict(rope_style=3), dict(rope_theta=0.0),
           dict(norm_kind=2),
           dict(rms_eps=-1.0), dict(n_kv_heads=0)]
    for over in bad:
        with pytest.raises(hc.HCacheError) as e:
            hc.validate_desc(good_desc(hc, **over))
        assert e.value.status == hc.HC_EINVAL, over
        assert str(e.value)


def read_chunk(store, seq, layer, c, d):
    import ctypes
    ptr, rows = store.chunk(seq, layer, c)
    buf = (ctypes.c_uint16 * (rows * d)).from_address(ptr)
    return np.frombuffer(buf, dtype=np.uint16).reshape(rows, d).copy()


def test_store_matches_oracle_model(hc):
    L, d, CT, T = 3, 16, 4, 11
    st = hc.Store(L, d, CT, capacity_chunks=64, pinned=False)
    ref = oracle.ChunkStore(L, d, CT)
    rng = np.random.default_rng(1)
    full = rng.integers(0, 65536, size=(L, T, d), dtype=np.uint16)
    # generation order: prefill of 5 tokens, then token by token, layer by layer
    steps = [(0, 5)] + [(t, t + 1) for t in range(5, T)]
    for a, b in steps:
        for l in range(L):
            rows = np.ascontiguousarray(full[l, a:b])
            st.append(7, l, rows, b - a)
            ref.append(7, l, rows)
    for l in range(L):
        assert st.tokens(7, l) == T == ref.n_tokens(7, l)
        for c in range(ref.n_chunks(7, l)):
            assert np.array_equal(read_chunk(st, 7, l, c, d), ref.chunk(7, l, c))
        with pytest.raises(hc.HCacheError) as e:
            st.chunk(7, l, ref.n_chunks(7, l))
        assert e.value.status == hc.HC_ERANGE
    # Figure 6: 2nd token, 2nd layer -> chunk (layer 1, 0), row 1
    assert np.array_equal(read_chunk(st, 7, 1, 0, d)[1], full[1, 1])
    # the arena is cut into rows of L chunk slots: chunk index c of every layer shares a row
    # (layer l at slot l of it), and a context's rows are consecutive while nothing interferes,
    # so a layer's chunks are exactly L slots apart -- one strided transfer per layer
    chunk_bytes = CT * d * 2
    p = [[st.chunk(7, l, c)[0] for c in range(3)] for l in range(L)]
    for c in range(3):
        assert p[1][c] - p[0][c] == chunk_bytes and p[2][c] - p[1][c] == chunk_bytes
    for l in range(L):
        assert p[l][1] - p[l][0] == L * chunk_bytes and p[l][2] - p[l][1] == L * chunk_bytes
    st.destroy()


def test_store_errors_and_reuse(hc):
    L, d, CT = 2, 8, 4
    st = hc.Store(L, d, CT, capacity_chunks=4, pinned=False)
    rows = np.zeros((8, d), dtype=np.uint16)
    with pytest.raises(hc.HCacheError) as e:        # layer 1 before layer 0
        st.append(1, 1, rows, 1)
    assert e.value.status == hc.HC_ESTATE
    with pytest.raises(hc.HCacheError) as e:
        st.append(1, 2, rows, 1)
    assert e.value.status == hc.HC_ERANGE
    st.append(1, 0, rows, 8)                        # 2 chunks
    st.append(1, 1, rows, 8)                        # 2 chunks -> arena full
    with pytest.raises(hc.HCacheError) as e:
        st.append(2, 0, rows, 1)
    assert e.value.status == hc.HC_ERANGE
    assert st.tokens(2, 0) == 0
    with pytest.raises(hc.HCacheError):
        st.drop(99)
    st.drop(1)
    assert st.tokens(1, 0) == 0
    st.append(2, 0, rows, 5)                        # reuses freed chunks
    assert st.tokens(2, 0) == 5
    assert st.chunk(2, 0, 1)[1] == 1                # tail chunk holds one row
    st.append(2, 0, rows, 0)                        # empty append is a no-op
    st.destroy()


def test_store_rows_stay_regular_under_interleaving_and_reuse(hc):
    """Four contexts appended in decode order (a few tokens at a time, taking turns), two of
    them dropped, two new ones appended into the holes: every context's chunks of a layer stay
    L slots apart in long runs (the spacing the strided loader needs), and every byte reads back."""
    L, d, CT, T = 4, 8, 4, 96
    n_idx = T // CT
    st = hc.Store(L, d, CT, capacity_chunks=L * (4 * n_idx + 8), pinned=False)
    rng = np.random.default_rng(4)
    data = {s: rng.integers(0, 65536, size=(L, T, d), dtype=np.uint16) for s in (1, 2, 3, 4, 5, 6)}

    def feed(ids):
        for a in range(0, T, 3):
            for s in ids:
                for l in range(L):
                    st.append(s, l, np.ascontiguousarray(data[s][l, a:a + 3]), 3)

    def runs(s, l):
        slots = [(st.chunk(s, l, c)[0] - st.chunk(1, 0, 0)[0]) // (CT * d * 2) for c in range(n_idx)]
        gaps = np.diff(slots)
        assert all((slots[c] - l) % L == 0 for c in range(n_idx))       # slot l of a row
        return 1 + int(np.sum(gaps != L))

    feed((1, 2, 3, 4))
    for s in (1, 2, 3, 4):
        assert max(runs(s, l) for l in range(L)) <= 3, "interleaved arrivals broke a context into many runs"
    st.drop(2)
    st.drop(4)
    feed((5, 6))
    for s in (1, 3, 5, 6):
        assert max(runs(s, l) for l in range(L)) <= 4
        for l in range(L):
            got = np.concatenate([read_chunk(st, s, l, c, d) for c in range(n_idx)])
            assert np.array_equal(got, data[s][l])
    st.destroy()


def test_store_bad_arguments(hc):
    for args in [(0, 8, 4, 4), (2, 0, 4, 4), (2, 8, 0, 4), (2, 8, 4, 0), (2, 12, 4, 4)]:
        with pytest.raises(hc.HCacheError) as e:
            hc.Store(*args, pinned=False)
        assert e.value.status == hc.HC_EINVAL


def test_create_fails_loudly_without_gpu(hc):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(hc.HCacheError) as e:
        hc.Context(good_desc(hc))
    assert e.value.status == hc.HC_EHIP


def test_partition_matches_oracle(hc):
    """The library's closed-form layer partition against the oracle (which is itself pinned to
    the brute-force optimum and to the schedules the paper prints)."""
    rng = np.random.default_rng(8)
    for _ in range(500):
        n = int(rng.integers(1, 129))
        io_h, c_h = float(rng.uniform(0.1, 3)), float(rng.uniform(0.1, 3))
        io_kv, c_tok = io_h * float(rng.uniform(1.01, 6)), c_h * float(rng.uniform(1.01, 20))
        l_h, l_o, comp = hc.partition_layers(n, io_h, io_kv, c_h, c_tok)
        want = oracle.partition_layers(n, io_h, io_kv, c_h, c_tok)
        assert (l_h, l_o, "kv" if comp == 0 else "re") == want
    assert hc.partition_layers(32, 1.0, 2.0, 1.1, 10.0) == (31, 1, 0)
    # the ceiling is the plain one: a quotient 8.4e-10 above 9 gives 10 layers, on both sides
    for c_h, want in ((2.0, 9), (2.0 - 2.0 ** -30, 10), (2.0 + 2.0 ** -30, 9)):
        assert hc.partition_layers(10, 1.0, 9.0, c_h, 50.0) == (want, 10 - want, 0)
        assert oracle.partition_layers(10, 1.0, 9.0, c_h, 50.0) == (want, 10 - want, "kv")
    for bad in [(0, 1, 1, 1, 1), (4, 0, 1, 1, 1), (4, 1, -1, 1, 1), (4, 1, 1, 0, 1), (4, 1, 1, 1, float("nan")),
                (4, 2, 1, 3, 9), (4, 1, 2, 3, 2)]:
        with pytest.raises(hc.HCacheError) as e:
            hc.partition_layers(*bad)
        assert e.value.status == hc.HC_EINVAL


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; asking the benchmark for more must say so and fail."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""


def test_header_is_plain_c_and_links(hc, tmp_path):
    """include/hcache.h compiles as pedantic C99 and a C program can call the library."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    libdir = os.path.dirname(hc.lib_path())
    exe = str(tmp_path / "cabi_smoke")
    rocm_lib = "/opt/rocm/lib"
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "cabi_smoke.c"), "-o", exe, "-L", libdir, "-lhcache",
           f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{rocm_lib}"]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    assert "hcache-mi355x" in res.stdout


def test_store_index_is_safe_across_threads(hc):
    """Appends, queries and drops of different contexts from several host threads at once."""
    import threading
    L, d, CT, per_ctx = 2, 64, 4, 40
    n_threads, rounds = 6, 30
    st = hc.Store(L, d, CT, capacity_chunks=n_threads * L * (per_ctx // CT) + 8, pinned=False)
    errors = []

    def worker(tid):
        try:
            rng = np.random.default_rng(tid)
            for r in range(rounds):
                sid = tid * 1000 + r
                rows = rng.integers(0, 65536, size=(per_ctx, d), dtype=np.uint16)
                for a in range(0, per_ctx, 10):
                    for l in range(L):
                        st.append(sid, l, np.ascontiguousarray(rows[a:a + 10]), 10)
                    st.tokens((tid + 1) % n_threads * 1000 + r, 0)      # someone else's context
                for l in range(L):
                    assert st.tokens(sid, l) == per_ctx
                    got = np.concatenate([read_chunk(st, sid, l, c, d) for c in range(per_ctx // CT)])
                    assert np.array_equal(got, rows)
                st.drop(sid)
        except Exception as e:                               # noqa: BLE001 - reported below
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    st.destroy()


def test_tile_map_covers_every_tile_once_and_balances_the_xcds(hc):
    """The kernel's slot -> tile map (the same function the kernel compiles, evaluated on the
    host): for a range of layer shapes and launch depths every tile of every layer belongs to
    exactly one slot, a slot's workgroup stays inside its XCD's super tiles (slot % 8), and over
    an eight-layer launch the XCDs differ by at most one super tile's worth of tiles."""
    import numpy as np
    shapes = [(1024, 8192), (4096, 2048), (7168, 2048), (5120, 1536), (5120, 1600), (192, 257),
              (128, 1), (640, 600), (1024, 32768), (384, 280)]
    for d_kv, n_tok in shapes:
        for n_layers in (1, 3, 8):
            shape, tiles = hc.diag_tile_map(d_kv, n_tok, n_layers)
            nf, nt, slots = shape["nf"], shape["nt"], shape["slots"]
            assert slots % 8 == 0 and shape["gf"] * shape["gt"] <= 32
            assert nf == 2 * (-(-d_kv // 128) * 128) // 256 and nt == -(-n_tok // 256)
            per_xcd = np.zeros(8, dtype=np.int64)
            for l in range(n_layers):
                t = tiles[l]
                real = t[:, 0] >= 0
                assert ((t[real, 0] < nf) & (t[real, 1] < nt)).all()
                flat = t[real, 0].astype(np.int64) * nt + t[real, 1]
                assert flat.size == nf * nt and np.unique(flat).size == nf * nt, (d_kv, n_tok, n_layers, l)
                # workgroup l * slots + w runs on XCD (l * slots + w) % 8 = w % 8
                per_xcd += np.bincount(np.nonzero(real)[0] % 8, minlength=8)
                # the tiles an XCD works on in one layer come from whole super tiles
                for x in range(8):
                    tx = t[real & (np.arange(slots) % 8 == x)]
                    supers = {(int(a) // shape["gf"], int(b) // shape["gt"]) for a, b in tx}
                    assert len(tx) <= len(supers) * shape["gf"] * shape["gt"]
            if n_layers == 8:
                assert per_xcd.max() - per_xcd.min() <= shape["gf"] * shape["gt"], (d_kv, n_tok, per_xcd)
    # a single-layer launch applies no rotation: slot w of layer 0 is the same in both
    one = hc.diag_tile_map(7168, 2048, 1)[1]
    many = hc.diag_tile_map(7168, 2048, 8)[1]
    assert (one[0] == many[0]).all() and not (many[1] == many[0]).all()


def test_split_plan_invariants(hc):
    """hc_diag_split_plan (host logic only).  Whenever a launch is split: its last round of 256
    workgroups would be at most half full; the whole tiles are the whole rows of token tiles
    that fit the full rounds and their slot grid is the one an unsplit launch of that many
    tokens gets; every share of a split loop is at least 8 x 64 channels; the workspace holds
    one slot per split workgroup (256 at most).  Mode 1 splits a subset of what mode 2 splits,
    in the same way, and only where its cost model (1.5 x the 64-channel steps of a whole tile against
    steps / ways + 0.143 x tiles x ways + 15) says so; mode 0 never splits."""
    for d_model in (256, 1024, 2048, 4096, 5120, 7168, 8192):
        nm = d_model // 64
        for d_kv in (64, 640, 1024, 5120, 7168):
            for n_tok in list(range(1, 4500, 173)) + [256, 1536, 1600, 2048, 8192, 16384]:
                p0, p1, p = (hc.diag_split_plan(d_model, d_kv, n_tok, m) for m in (0, 1, 2))
                nf, nt = p["nf"], p["nt"]
                assert nf == 2 * (-(-d_kv // 128) * 128) // 256 and nt == -(-n_tok // 256)
                unsplit = dict(p, split=0, nt_main=nt, n_tail=0, n_split=1, main_slots=0, fixup_workgroups=0)
                assert p0 == unsplit and p1 in (unsplit, p)
                if not p["split"]:
                    assert p == unsplit
                    continue
                rem = nf * nt % 256
                assert 0 < rem <= 128
                assert nf * p["nt_main"] <= nf * nt - rem                   # whole tiles stay within the full rounds
                assert nf * (p["nt_main"] + 1) > nf * nt - rem              # ... and no further row would
                assert p["n_tail"] == nf * (nt - p["nt_main"]) > 0
                assert 2 <= p["n_split"] <= 16 and p["n_tail"] * p["n_split"] <= 256
                assert nm // p["n_split"] >= 8
                assert p["fixup_workgroups"] == 4 * p["n_tail"]
                if p["nt_main"]:
                    assert p["main_slots"] == hc.diag_tile_map(d_kv, 256 * p["nt_main"], 1)[0]["slots"]
                else:
                    assert p["main_slots"] == 0
                cost = nm / p["n_split"] + 0.143 * p["n_tail"] * p["n_split"] + 15
                if abs(cost - 1.5 * nm) > 1e-3:
                    assert p1["split"] == (cost < 1.5 * nm), (d_model, d_kv, n_tok, cost)
    p = hc.diag_split_plan(5120, 5120, 1600)                                # 40 x 7 tiles
    assert (p["split"], p["nt_main"], p["n_tail"], p["n_split"], p["main_slots"]) == (1, 6, 40, 4, 256)
    assert hc.diag_split_plan(4096, 1024, 8192, 2)["split"] == 0            # 8 x 32 tiles: exactly one round
    assert hc.diag_split_plan(5120, 5120, 1536, 2)["split"] == 0            # 240 of 256: full enough
    assert hc.diag_split_plan(1024, 640, 600)["split"] == 0                 # narrow model: does not pay
    assert hc.diag_split_plan(1024, 640, 600, 2)["n_split"] == 2
    with pytest.raises(hc.HCacheError):
        hc.diag_split_plan(100, 64, 10)
    with pytest.raises(hc.HCacheError):
        hc.diag_split_plan(1024, 64, 10, 3)
