"""Host side of libapar without a GPU: the library loads, exports what apar.h declares, and its
bookkeeping and plan builder (run on dry-run pools, which never touch a device) match the ledger."""
import os
import re

import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import HeadConfig, make_config, manual_tree, tiny_tree
from oracle import BlockLedger

from harness import (PlanTablesOnDevice, blocks_upper_bound, books_equal, check_plan_covers_tables, nested_wide_tree, pool_for, random_forest,
                     replay_trace)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "apar.h")).read()
    declared = list(dict.fromkeys(re.findall(r"APAR_API\s+(?:const\s+char\*|int)\s+(apar_[a-z_0-9]+)\s*\(", hdr)))
    assert len(declared) >= 20
    assert set(declared) <= set(ap.exported_symbols())
    for name in ("apar_pool_create", "apar_fork", "apar_append_kv", "apar_decode_attention", "apar_free_thread"):
        assert name in declared
    assert ap.apar_status_string(0) == "ok" and "blocks" in ap.apar_status_string(-3)


def test_tiny_books_match_ledger_after_every_op():
    w = tiny_tree()
    with pool_for(w, 8, dry_run=True) as pool:
        led = BlockLedger(8)
        live, _ = replay_trace(w, pool, led, dry_run=True, check_each=True)
        assert live == [1, 2, 3]
        assert [ap.apar_thread_block_table(pool.handle, t) for t in live] == [[0, 2], [0, 3], [0, 1, 4]]
        ap.apar_decode_attention(pool.handle, None, live, None)
        info = ap.apar_last_plan_info(pool.handle)
        assert info.unique_blocks == 5 and info.path_tokens == 97
        check_plan_covers_tables(pool.handle, live, 2)


@pytest.mark.parametrize("name,n_req", [("mha64", 6), ("ht256", 24), ("gqa1024", 3), ("spec128", 10)])
def test_config_books_and_plans(name, n_req):
    w = make_config(name, n_requests=n_req)
    N = blocks_upper_bound(w)
    with pool_for(w, N, dry_run=True) as pool:
        led = BlockLedger(N)
        live, _ = replay_trace(w, pool, led, dry_run=True)
        books_equal(pool.handle, led)
        led.check_invariants()
        for chunk in (1, 8, 64, 512):
            ap.apar_set_chunk_blocks(pool.handle, chunk)
            ap.apar_decode_attention(pool.handle, None, live, None)
            res = check_plan_covers_tables(pool.handle, live, w.heads.n_kv_heads, w.heads.n_q_heads // w.heads.n_kv_heads)
            groups_extra = res["unit_block_reads"] - res["unique_blocks"]
            # a block is read once per workgroup that holds rows for it; only runs shared by more
            # than 64 rows are split over several workgroups
            assert groups_extra >= 0
            if w.heads.n_q_heads == w.heads.n_kv_heads:
                assert groups_extra == 0
            if chunk == 512 and name != "gqa1024":
                # whole trees fit one unit: nothing is left to merge
                assert res["partial_rows"] == 0 and res["direct_threads"] == len(live)
        info = ap.apar_last_plan_info(pool.handle)
        e = w.heads.elem_bytes
        assert info.algorithmic_bytes == info.unique_tokens * w.heads.kv_bytes_per_token + \
            2 * len(live) * w.heads.n_q_heads * w.heads.head_dim * e
        # a shuffled and partly repeated list is planned just as well
        rng = np.random.default_rng(0)
        some = [int(x) for x in rng.permutation(live)[: max(2, len(live) // 2)]]
        some += some[:2]
        ap.apar_decode_attention(pool.handle, None, some, None)
        check_plan_covers_tables(pool.handle, some, w.heads.n_kv_heads, w.heads.n_q_heads // w.heads.n_kv_heads)
        # the speculative call plans 5 rows per thread and head
        ap.apar_decode_attention_spec(pool.handle, None, None, None, None, 5, live, None)
        check_plan_covers_tables(pool.handle, live, w.heads.n_kv_heads, 5 * w.heads.n_q_heads // w.heads.n_kv_heads)
        # releasing everything returns every block
        for t in live:
            ap.apar_free_thread(pool.handle, t)
            led.free(t)
        books_equal(pool.handle, led)
        assert ap.apar_pool_stats(pool.handle).free_blocks == N


def test_random_interleavings_match_ledger():
    rng = np.random.default_rng(5)
    for trial in range(25):
        N = int(rng.integers(6, 40))
        heads = HeadConfig(2, 1, 64, "f32")
        with ap.Pool(2, 1, 64, "f32", N, max_threads=64, dry_run=True) as pool:
            h = pool.handle
            led = BlockLedger(N, max_threads=64)
            assert ap.apar_thread_create(h) == led.create()
            for _ in range(80):
                live = led.live()
                op = rng.choice(["append", "append", "batch", "fork", "free", "create"])
                t = int(rng.choice(live)) if live else -1
                if op == "create" or not live:
                    try:
                        want = led.create()
                    except Exception:
                        with pytest.raises(ap.AparError) as ei:
                            ap.apar_thread_create(h)
                        assert ei.value.status == -4
                        continue
                    assert ap.apar_thread_create(h) == want
                elif op == "append":
                    n = int(rng.choice([1, 3, 15, 16, 17, 40]))
                    try:
                        led.append(t, n)
                    except Exception:
                        with pytest.raises(ap.AparError) as ei:
                            ap.apar_append_kv(h, t, None, None, n)
                        assert ei.value.status == -3
                    else:
                        ap.apar_append_kv(h, t, None, None, n)
                elif op == "batch":
                    ts = [int(x) for x in rng.choice(live, size=int(rng.integers(1, 7)))]
                    try:
                        led.append_batch(ts)
                    except Exception:
                        with pytest.raises(ap.AparError) as ei:
                            ap.apar_append_kv_batch(h, ts, None, None)
                        assert ei.value.status == -3
                    else:
                        ap.apar_append_kv_batch(h, ts, None, None)
                elif op == "fork":
                    n = int(rng.integers(1, 4))
                    try:
                        want = led.fork(t, n)
                    except Exception:
                        with pytest.raises(ap.AparError) as ei:
                            ap.apar_fork(h, t, n)
                        assert ei.value.status == -4
                    else:
                        assert ap.apar_fork(h, t, n) == want
                else:
                    led.free(t)
                    ap.apar_free_thread(h, t)
                books_equal(h, led)
            led.check_invariants()
            listed = [t for t in led.live() if led.len[t] > 0]
            if listed:
                ap.apar_decode_attention(h, None, listed, None)
                check_plan_covers_tables(h, listed, 1, 2)


def test_error_codes_and_noops():
    with ap.Pool(4, 2, 64, "f32", 4, max_threads=3, dry_run=True) as pool:
        h = pool.handle
        t = ap.apar_thread_create(h)

        def status(fn, *a):
            with pytest.raises(ap.AparError) as ei:
                fn(*a)
            return ei.value.status

        assert status(ap.apar_fork, h, t, 0) == -1
        assert status(ap.apar_fork, h, 7, 1) == -2
        assert status(ap.apar_fork, h, t, 3) == -4  # would issue ids 1..3 with max_threads = 3
        assert status(ap.apar_decode_attention, h, None, [t], None) == -1  # empty thread
        assert status(ap.apar_append_kv, h, t, None, None, 65) == -3  # needs 5 blocks of 4
        assert ap.apar_pool_stats(h).free_blocks == 4 and ap.apar_thread_len(h, t) == 0
        ap.apar_append_kv(h, t, None, None, 0)
        ap.apar_decode_attention(h, None, [], None)
        ap.apar_append_kv(h, t, None, None, 64)
        assert status(ap.apar_append_kv, h, t, None, None, 1) == -3
        (c,) = ap.apar_fork(h, t, 1)
        ap.apar_free_thread(h, t)
        assert status(ap.apar_free_thread, h, t) == -2
        assert status(ap.apar_thread_len, h, t) == -2
        assert status(ap.apar_append_kv, h, t, None, None, 1) == -2
        assert status(ap.apar_decode_attention, h, None, [c, t], None) == -2
        assert status(ap.apar_block_refcount, h, 4) == -1
        assert ap.apar_thread_block_table(h, c) == [0, 1, 2, 3]
        ap.apar_free_thread(h, c)
        assert ap.apar_pool_stats(h).free_blocks == 4
    for bad in (dict(block_size=8), dict(n_q_heads=3), dict(num_blocks=0), dict(num_blocks=(1 << 26) + 1), dict(dtype=7)):
        kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=64, block_size=16, dtype=0, max_threads=8, num_blocks=4,
                  softmax_scale=0.0)
        kw.update(bad)
        with pytest.raises(ap.AparError) as ei:
            ap.apar_pool_create(ap.AparPoolConfig(**kw), None)
        assert ei.value.status == -1
    with pytest.raises(ap.AparError) as ei:
        ap.apar_pool_create(ap.AparPoolConfig(4, 4, 96, 16, 1, 8, 4, 0.0), None)
    assert ei.value.status == -6


@pytest.mark.parametrize("n_q,n_kv,fan,n_cand", [
    (4, 4, 70, 1),     # 71 rows per kv head share the root: two 16-row tiles per wavefront
    (4, 4, 130, 1),    # more rows than one workgroup holds: the root stands alone, chunks of 128 rows
    (4, 4, 300, 1),
    (8, 1, 9, 1),      # 8 rows per thread: 2 threads per tile
    (8, 1, 30, 1),
    (8, 1, 40, 1),
    (8, 1, 3, 5),      # 40 rows per thread: three slices of 14 rows, one row group per tile
    (8, 1, 6, 5),
])
def test_wide_sharing_groups_use_more_row_tiles(n_q, n_kv, fan, n_cand):
    # a root of 40 tokens with `fan` children, every second child with two children of its own
    parents, lens = [-1], [40]
    for c in range(fan):
        parents.append(0)
        lens.append(5 + (c * 7) % 50)
        if c % 2:
            kid = len(parents) - 1
            parents += [kid, kid]
            lens += [3 + c % 20, 17]
    w = manual_tree(parents, lens, HeadConfig(n_q, n_kv, 128, "bf16"))
    N = blocks_upper_bound(w)
    rpt = n_cand * n_q // n_kv
    with pool_for(w, N, dry_run=True) as pool:
        live, _ = replay_trace(w, pool, None, dry_run=True)
        for chunk, matrix_rows, inline in ((2, 64, True), (512, 64, True), (2, 0, True), (512, 0, True), (512, 1, True),
                                           (2, 64, False), (512, 0, False), (512, 1, False)):
            ap.apar_set_chunk_blocks(pool.handle, chunk)
            ap.apar_set_matrix_units(pool.handle, matrix_rows, 1)
            ap.apar_set_inline_shared(pool.handle, inline)
            if n_cand == 1:
                ap.apar_decode_attention(pool.handle, None, live, None)
            else:
                ap.apar_decode_attention_spec(pool.handle, None, None, None, None, n_cand, live, None)
            res = check_plan_covers_tables(pool.handle, live, n_kv, rpt)
            wgs = np.array(ap.apar_last_plan_export(pool.handle, ap.APAR_PLAN_WORKGROUPS)).reshape(-1, 32)
            n_sl = -(-rpt // 16)
            cap = 16 // -(-rpt // n_sl)
            groups = len(live) * n_sl
            if chunk == 512 and groups <= 8 * cap:
                # the whole tree is one unit with the fewest row tiles that hold it
                want = 1 if groups <= 4 * cap else 2
                assert res["partial_rows"] == 0 and len(wgs) == 1 and wgs[0][3] & 255 == want
            if groups > 8 * cap:
                to_matrix = matrix_rows and len(live) * rpt >= matrix_rows
                if inline and not to_matrix and (chunk == 512 or res["partial_rows"] == 0):
                    # the tree is cut by rank: full units of consecutive threads, each reading the segments above
                    # its threads again (the root by every unit), all direct, nothing to merge
                    assert res["partial_rows"] == 0 and res["direct_threads"] == len(live)
                    assert res["unit_block_reads"] > res["unique_blocks"] and all(x & 255 in (1, 2) for x in wgs[:, 3])
                    per_unit = max(1, 8 * cap // n_sl)
                    assert len(wgs) == -(-len(live) // per_unit)  # as few units as the rows allow
                else:
                    # the root stands alone: as matrix units (marked 32) when its holders bring enough rows
                    assert res["partial_rows"] > 0 and wgs[0][3] & 255 == (32 if to_matrix else 2)


@pytest.mark.parametrize("n_cand", [1, 5])
def test_nested_wide_groups_are_inlined_or_stand_alone(n_cand):
    w = nested_wide_tree(HeadConfig(2, 2, 128, "bf16"))
    N = blocks_upper_bound(w) + 600
    with pool_for(w, N, dry_run=True) as pool:
        h = pool.handle
        live, _ = replay_trace(w, pool, None, dry_run=True)
        # 200 threads forked off one leaf and listed before they get rows of their own: they all end at a
        # segment that is shared by more rows than one unit carries
        kids = ap.apar_fork(h, live[0], 200)
        listed = live + kids

        def plan():
            if n_cand == 1:
                ap.apar_decode_attention(h, None, listed, None)
            else:
                ap.apar_decode_attention_spec(h, None, None, None, None, n_cand, listed, None)
            return check_plan_covers_tables(h, listed, 2, n_cand)

        ap.apar_set_matrix_units(h, 0, 0)
        res = plan()  # the whole tree is cut by rank into direct units: nothing to merge
        assert res["partial_rows"] == 0 and res["direct_threads"] == len(listed)
        ap.apar_set_inline_shared(h, False)
        off = plan()
        assert off["partial_rows"] > 0 and off["unit_block_reads"] <= res["unit_block_reads"]
        ap.apar_set_inline_shared(h, True)
        # a matrix-kernel threshold that only a segment inside the tree meets changes nothing: the root decides
        ap.apar_set_matrix_units(h, 64, 8)
        assert plan() == res
        # a root that meets it stands alone on the matrix kernel, and what is wide below it follows
        ap.apar_set_matrix_units(h, 64, 2)
        assert plan()["partial_rows"] > 0
        ap.apar_set_matrix_units(h, 0, 0)
        # a unit cap too small for the paths of a unit's threads: the root stands alone, and so does everything wide below it
        ap.apar_set_chunk_blocks(h, 4)
        res = plan()
        assert res["partial_rows"] > 0


@pytest.mark.parametrize("seed", range(24))
def test_random_forest_plans_cover_every_table(seed):
    """Planner fuzz on bookkeeping-only pools: random forests, head grouping, candidates, unit caps and policy
    knobs; every plan must show every row group exactly its thread's blocks, once."""
    rng = np.random.default_rng(5000 + seed)
    n_kv = int(rng.choice([1, 2]))
    group = int(rng.choice([1, 2, 4, 8, 16]))
    parents, segs = random_forest(rng, int(rng.integers(1, 4)), int(rng.integers(8, 260)))
    w = manual_tree(parents, segs, HeadConfig(n_kv * group, n_kv, 128, "bf16"), seed=seed)
    N = blocks_upper_bound(w) + 64
    with pool_for(w, N, dry_run=True) as pool:
        h = pool.handle
        live, _ = replay_trace(w, pool, None, dry_run=True)
        # some threads forked and listed before they get rows of their own
        extra = []
        for t in rng.choice(live, size=min(3, len(live)), replace=False):
            extra += ap.apar_fork(h, int(t), int(rng.integers(1, 40)))
        listed = [int(x) for x in rng.permutation(live + extra)]
        for _ in range(3):
            ap.apar_set_chunk_blocks(h, int(rng.choice([1, 2, 5, 16, 512])))
            ap.apar_set_matrix_units(h, int(rng.choice([0, 1, 64])), int(rng.choice([1, 3, 128])))
            ap.apar_set_inline_shared(h, bool(rng.integers(0, 2)))
            C = int(rng.choice([1, 1, 2, 4]))
            if C * group > 64:
                C = 1
            if C == 1 and rng.integers(0, 2):
                ap.apar_decode_attention(h, None, listed, None)
            else:
                ap.apar_decode_attention_spec(h, None, None, None, None, C, listed, None)
            check_plan_covers_tables(h, listed, n_kv, C * group)


@pytest.mark.parametrize("seed", range(12))
def test_plans_carried_over_a_decode_loop_cover_every_table(seed):
    """Decode loops on bookkeeping-only pools over random forests (Alg. 1's per-step loop: the same threads, each
    a row longer, a few replaced by a thread forked from them): from the second step on the plan is the previous
    one brought up to date, and after every step it must show every row group exactly its thread's blocks with
    the right fill counts, like a plan built afresh.  Planner knobs, head grouping and candidate counts vary; some
    loops commit several rows per step, fork threads that are not listed (their parent's next row then goes to a
    copy-on-write copy) or grow a thread by several blocks at once (which a carried plan cannot follow: that call
    builds a new one)."""
    rng = np.random.default_rng(9000 + seed)
    n_kv = int(rng.choice([1, 2]))
    group = int(rng.choice([1, 2, 4, 8, 16]))
    parents, segs = random_forest(rng, int(rng.integers(1, 4)), int(rng.integers(8, 120)))
    w = manual_tree(parents, segs, HeadConfig(n_kv * group, n_kv, 128, "bf16"), seed=seed)
    steps = 40
    n_leaves = len(w.leaves())
    N = blocks_upper_bound(w) + n_leaves * (steps // 4 + 8) + 256
    with pool_for(w, N, dry_run=True, max_threads=len(parents) + n_leaves * (steps + 8) + 64) as pool:
        h = pool.handle
        live, _ = replay_trace(w, pool, None, dry_run=True)
        listed = [int(x) for x in rng.permutation(live)]
        ap.apar_set_chunk_blocks(h, int(rng.choice([2, 5, 16, 512])))
        ap.apar_set_matrix_units(h, int(rng.choice([0, 1, 64])), int(rng.choice([1, 3, 128])))
        ap.apar_set_inline_shared(h, bool(rng.integers(0, 2)))
        C = int(rng.choice([1, 1, 2, 4]))
        if C * group > 64:
            C = 1
        spec = C > 1 or bool(rng.integers(0, 2))
        rough = seed % 3 == 2  # loops with the changes a carried plan cannot follow
        expected_built = 1
        on_device = PlanTablesOnDevice(h)
        for step in range(steps):
            changed_shape = False
            for pos in range(len(listed)):
                coin = rng.integers(0, 40)
                if coin == 0:    # a thread finishes and one forked from it carries on in its place
                    (child,) = ap.apar_fork(h, listed[pos], 1)
                    ap.apar_free_thread(h, listed[pos])
                    listed[pos] = child
                elif coin == 1:  # forked, the fork not listed
                    ap.apar_fork(h, listed[pos], 1)
                elif coin == 2 and rough and step > 0:
                    ap.apar_append_kv(h, listed[pos], None, None, 33)
                    changed_shape = True
            if spec and rng.integers(0, 2):
                masks = rng.integers(0, 1 << min(C, 3), size=len(listed)).astype(np.uint8)
                ap.apar_commit_candidates(h, listed, None, None, C, masks)
            else:
                ap.apar_append_kv_batch(h, listed, None, None)
            if spec:
                ap.apar_decode_attention_spec(h, None, None, None, None, C, listed, None)
            else:
                ap.apar_decode_attention(h, None, listed, None)
            check_plan_covers_tables(h, listed, n_kv, C * group)
            on_device.follow()
            expected_built += 1 if changed_shape else 0
        built, carried = ap.apar_plan_counts(h)
        assert built + carried == steps
        # besides the calls that had to, a new plan is only built when a list has no free entry left behind it
        assert expected_built <= built <= expected_built + 3, (built, carried, expected_built)


def _sanitizer_build(tmp_path, name, sources, extra=()):
    """Compiles tests/native/<name>.cpp with the given library sources as plain host C++ under the address and
    undefined-behaviour sanitizers; returns the executable, or skips when the toolchain cannot."""
    import shutil
    import subprocess

    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2401_06761_amd", "csrc")
    exe = str(tmp_path / name)
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(root, "include"), "-I" + csrc,
           os.path.join(root, "tests", "native", name + ".cpp")] + [os.path.join(csrc, f) for f in sources] + \
          list(extra) + ["-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitize" in built.stderr:
        pytest.skip("this g++ has no sanitizer runtime")
    assert built.returncode == 0, built.stderr[-2000:]
    return exe


def _run_sanitized(exe, count, what):
    import subprocess

    ran = subprocess.run([exe, "0", str(count)], capture_output=True, text=True, timeout=900)
    if "ASan runtime does not come first" in ran.stderr:
        pytest.skip("a preloaded library keeps the sanitizer runtime from starting here")
    assert ran.returncode == 0 and f"ok: {count} {what}" in ran.stdout, (ran.stdout + ran.stderr)[-3000:]


def test_plan_builder_under_sanitizers(tmp_path):
    """The plan builder compiled as plain host C++ with the address and undefined-behaviour sanitizers and
    fuzzed over random forests, geometries and policy knobs (tests/native/fuzz_plan.cpp checks coverage too)."""
    exe = _sanitizer_build(tmp_path, "fuzz_plan", ["plan.cpp"])
    _run_sanitized(exe, 60, "forests")


def test_pool_controller_and_server_under_sanitizers(tmp_path):
    """The library's host side (allocator, copy-on-write, commits, plans, Algorithm 1 controller, serving loop)
    on bookkeeping-only pools, under the sanitizers (leak detection included), driven by random operation
    sequences on pools small enough to run out of blocks (tests/native/fuzz_pool.cpp; the kernels' launchers
    are stubs there)."""
    if not os.path.exists("/opt/rocm/lib/libamdhip64.so"):
        pytest.skip("no HIP runtime to link the host side against")
    exe = _sanitizer_build(tmp_path, "fuzz_pool", ["plan.cpp", "apar_pool.cpp", "controller.cpp"],
                           extra=["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    _run_sanitized(exe, 30, "sequences")


def test_commit_candidates_books_and_errors():
    # dry-run pools: the commit leaves the same books as one batched append per accepted candidate
    heads = HeadConfig(4, 2, 64, "f32")
    w = manual_tree([-1, 0, 0, 2, 2, -1], [30, 16, 9, 1, 25, 3], heads)
    N = blocks_upper_bound(w) + 8
    rng = np.random.default_rng(5)
    with pool_for(w, N, dry_run=True) as pool:
        led = BlockLedger(N)
        live, _ = replay_trace(w, pool, led, dry_run=True)
        for C in (1, 5, 8):
            masks = rng.integers(0, 1 << C, size=len(live)).astype(np.uint8)
            masks[0] = 0
            ap.apar_commit_candidates(pool.handle, live, None, None, C, masks)
            led.commit_candidates(live, masks)
            books_equal(pool.handle, led)
        # a thread may repeat
        ap.apar_commit_candidates(pool.handle, [live[1], live[1]], None, None, 3, [0b101, 0b010])
        led.commit_candidates([live[1], live[1]], [0b101, 0b010])
        books_equal(pool.handle, led)
        for bad in (lambda: ap.apar_commit_candidates(pool.handle, live[:1], None, None, 3, [0b1000]),
                    lambda: ap.apar_commit_candidates(pool.handle, live[:1], None, None, 9, [1]),
                    lambda: ap.apar_commit_candidates(pool.handle, live[:1], None, None, 0, [0])):
            with pytest.raises(ap.AparError) as e:
                bad()
            assert e.value.status == -1
        with pytest.raises(ap.AparError) as e:
            ap.apar_commit_candidates(pool.handle, [10 ** 6], None, None, 2, [1])
        assert e.value.status == -2
        books_equal(pool.handle, led)
    # all or nothing when the pool runs out
    with ap.Pool(4, 2, 64, "f32", 3, dry_run=True) as pool:
        led = BlockLedger(3)
        t = ap.apar_thread_create(pool.handle)
        led.create()
        ap.apar_append_kv(pool.handle, t, None, None, 30)
        led.append(t, 30)
        kid = ap.apar_fork(pool.handle, t, 1)[0]
        led.fork(t, 1)
        # t needs a copy of the shared tail (1 block) and kid another copy plus a new block: 3 > 1 free
        with pytest.raises(ap.AparError) as e:
            ap.apar_commit_candidates(pool.handle, [t, kid], None, None, 5, [0b00001, 0b11111])
        assert e.value.status == -3
        books_equal(pool.handle, led)
        ap.apar_commit_candidates(pool.handle, [t, kid], None, None, 5, [0b00001, 0b00000])
        led.commit_candidates([t, kid], [1, 0])
        books_equal(pool.handle, led)


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (8, 2), (8, 1), (16, 1)])
def test_prefill_plans_show_every_query_its_causal_path(n_q, n_kv):
    from harness import check_prefill_plan

    heads = HeadConfig(n_q, n_kv, 128, "bf16")
    # segment lengths around every block boundary, a long root (several workgroups), nested forks
    parents = [-1, 0, 0, 1, 1, 2, -1, 6, 6]
    segs = [300, 15, 16, 17, 1, 33, 70, 130, 2]
    w = manual_tree(parents, segs, heads)
    N = blocks_upper_bound(w)
    with pool_for(w, N, dry_run=True) as pool:
        live, nodes = replay_trace(w, pool, None, dry_run=True)
        lens = [ap.apar_thread_len(pool.handle, t) for t in live]
        # every live thread's own segment
        m = [w.nodes[i].seg_len for i in nodes]
        ap.apar_prefill_attention(pool.handle, None, live, m, None)
        check_prefill_plan(pool.handle, live, m, n_q // n_kv)
        info = ap.apar_last_plan_info(pool.handle)
        assert info.path_tokens == sum(mi * (L - mi) + mi * (mi + 1) // 2 for mi, L in zip(m, lens))
        # whole paths, single tokens, a thread listed twice
        for m2 in (lens, [1] * len(live), [min(L, 20) for L in lens]):
            ap.apar_prefill_attention(pool.handle, None, live, m2, None)
            check_prefill_plan(pool.handle, live, m2, n_q // n_kv)
        ap.apar_prefill_attention(pool.handle, None, [live[0], live[0]], [3, lens[0]], None)
        check_prefill_plan(pool.handle, [live[0], live[0]], [3, lens[0]], n_q // n_kv)
        for bad_m in ([0] + [1] * (len(live) - 1), [lens[0] + 1] + [1] * (len(live) - 1)):
            with pytest.raises(ap.AparError) as e:
                ap.apar_prefill_attention(pool.handle, None, live, bad_m, None)
            assert e.value.status == -1


def test_prefill_needs_a_group_size_that_divides_16():
    with ap.Pool(6, 2, 128, "bf16", 8, dry_run=True) as pool:
        t = ap.apar_thread_create(pool.handle)
        ap.apar_append_kv(pool.handle, t, None, None, 5)
        with pytest.raises(ap.AparError) as e:
            ap.apar_prefill_attention(pool.handle, None, [t], [5], None)
        assert e.value.status == -6


def test_prefill_kernel_knob_checks_its_argument_and_dry_runs_stay_on_row_tiles():
    with ap.Pool(4, 2, 128, "bf16", 8, dry_run=True) as pool:
        h = pool.handle
        for bad in ((-1, 1), (1, -1)):
            with pytest.raises(ap.AparError) as e:
                ap.apar_set_matrix_units(h, *bad)
            assert e.value.status == -1
        assert ap.apar_last_prefill_kernel(h) == 0
        for bad in (-1, 3):
            with pytest.raises(ap.AparError) as e:
                ap.apar_set_prefill_kernel(h, bad)
            assert e.value.status == -1
        t = ap.apar_thread_create(h)
        ap.apar_append_kv(h, t, None, None, 40)
        for which in (ap.APAR_PREFILL_AUTO, ap.APAR_PREFILL_ROW_TILES, ap.APAR_PREFILL_MATRIX):
            ap.apar_set_prefill_kernel(h, which)
            ap.apar_prefill_attention(h, None, [t], [40], None)
            # a dry run builds (and exports) the row-tile plan whatever the knob says
            assert ap.apar_last_prefill_kernel(h) == ap.APAR_PREFILL_ROW_TILES
            assert ap.apar_last_plan_info(h).path_tokens == 40 * 41 // 2


def test_empty_calls_are_no_ops_and_gather_checks_its_arguments():
    with ap.Pool(4, 2, 64, "f32", 8, dry_run=True) as pool:
        h = pool.handle
        t = ap.apar_thread_create(h)
        ap.apar_append_kv(h, t, None, None, 3)
        before = ap.apar_pool_stats(h).used_blocks
        ap.apar_commit_candidates(h, [], None, None, 5, [])
        ap.apar_append_kv_gather(h, [], [], None, None)
        ap.apar_prefill_attention(h, None, [], [], None)
        ap.apar_decode_attention(h, None, [], None)
        assert ap.apar_pool_stats(h).used_blocks == before and ap.apar_thread_len(h, t) == 3
        ap.apar_append_kv_gather(h, [t, t], [7, 0], None, None)
        assert ap.apar_thread_len(h, t) == 5
        with pytest.raises(ap.AparError) as e:
            ap.apar_append_kv_gather(h, [t], [-1], None, None)
        assert e.value.status == -1
        with pytest.raises(ap.AparError) as e:
            ap.apar_append_kv_gather(h, [99], [0], None, None)
        assert e.value.status == -2
        assert ap.apar_thread_len(h, t) == 5
