"""Shared test plumbing: replay one op trace on the library, the ledger and the dense oracle."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

import paper_2401_06761_amd as ap
from apar_workloads import build_trace, manual_tree, node_kv
from oracle import BlockLedger, DenseThreads


def to_dev(x: np.ndarray, dtype: str, device="cuda:0"):
    """fp32 numpy values (already representable in `dtype`) -> GPU tensor of the pool dtype."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
    return t if dtype == "f32" else t.to(torch.bfloat16)


def to_host(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


# bf16 pools: the bound the task states (max abs 2e-2) says little where outputs are small, so every bf16
# comparison also holds the error to the size of the outputs compared.  An output element is rounded to bf16
# once (relative 2^-8) and the probabilities once before the P.V product (2^-8 each, averaging out over the
# row): 2^-6 of the largest expected magnitude leaves a factor of about three over what is observed and is
# failed by an output of zeros, by a row of another thread and by a missing or foreign block.
REL_BF16 = 2.0 ** -6


def assert_close(got: np.ndarray, want: np.ndarray, dtype: str, what: str = "") -> float:
    """max abs error of got against want (fp64 arrays), asserted against both bounds; returns it."""
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = float(np.abs(got - want).max())
    if dtype == "f32":
        assert err <= 1e-5, f"{what}: max abs err {err}"
    else:
        top = float(np.abs(want).max())
        assert err <= 2e-2, f"{what}: max abs err {err}"
        assert err <= REL_BF16 * top, f"{what}: max abs err {err} against outputs of magnitude {top}"
    return err


# Values that say which token they belong to (for checks with a zero query, whose output is the plain mean of
# the V rows on a thread's root path).  Per token id, 128 channels: 0..23 the id's bits, 64..87 their
# complements, 40..63 twenty-four pseudo-random signs of the id (+-1, balanced, so that their means are small
# and bf16 resolves a change of a few counts at any path length); 32..39 and 96..103 are left for the caller
# (the kv head's bits).  Sums of these values over up to 2^24 rows are exact in fp32.
N_ID_BITS = 24
_HASH_MULT = np.array([0x9E3779B1 + 2 * 0x632BE5AB * j for j in range(24)], dtype=np.uint64)


def id_channels(ids: np.ndarray) -> np.ndarray:
    ids = np.asarray(ids, dtype=np.int64)
    out = np.zeros((len(ids), 128), dtype=np.float32)
    bits = ((ids[:, None] >> np.arange(N_ID_BITS)) & 1).astype(np.float32)
    out[:, :N_ID_BITS] = bits
    out[:, 64:64 + N_ID_BITS] = 1.0 - bits
    mixed = ((ids[:, None].astype(np.uint64) + np.uint64(1)) * _HASH_MULT[None, :]) & np.uint64(0xFFFFFFFF)
    mixed ^= mixed >> np.uint64(15)
    mixed = (mixed * np.uint64(0x2C1B3C6D)) & np.uint64(0xFFFFFFFF)
    out[:, 40:64] = 1.0 - 2.0 * ((mixed >> np.uint64(13)) & np.uint64(1)).astype(np.float32)
    return out


def books_equal(handle, led: BlockLedger, check_blocks: Optional[Sequence[int]] = None) -> None:
    """Block tables, lengths, refcounts and counters of the library against the ledger, bit-exact."""
    for t in led.live():
        assert ap.apar_thread_len(handle, t) == led.len[t], f"len of thread {t}"
        assert ap.apar_thread_block_table(handle, t) == led.table[t], f"table of thread {t}"
    blocks = range(led.N) if check_blocks is None else check_blocks
    for b in blocks:
        assert ap.apar_block_refcount(handle, b) == led.ref[b], f"refcount of block {b}"
    st = ap.apar_pool_stats(handle)
    assert st.used_blocks == led.used_blocks() and st.free_blocks == led.free_blocks()
    assert st.live_threads == len(led.live()) and st.cow_copies == led.cow_copies
    assert st.threads_issued == led.next_tid
    assert st.bytes_resident == led.used_blocks() * st.block_bytes
    assert st.bytes_vanilla == led.vanilla_blocks() * st.block_bytes


def replay_trace(w, pool: "ap.Pool", led: Optional[BlockLedger] = None, dense: Optional[DenseThreads] = None,
                 dry_run: bool = False, dense_nodes: Optional[set] = None, check_each: bool = False, kv_of=node_kv):
    """Runs build_trace(w) on the library and, if given, on the ledger and the dense oracle.
    kv_of(w, node) gives the K and V rows of a node's segment (the seeded recipe unless a test brings its own).
    Returns (live thread ids ascending, their node indices)."""
    ops, live, live_nodes = build_trace(w)
    h = pool.handle
    for op in ops:
        if op.kind == "create":
            assert ap.apar_thread_create(h) == op.tid
            if led is not None:
                assert led.create() == op.tid
            if dense is not None:
                assert dense.create() == op.tid
        elif op.kind == "append":
            if dry_run:
                ap.apar_append_kv(h, op.tid, None, None, op.n_tokens)
            else:
                k, v = kv_of(w, op.node)
                ap.apar_append_kv(h, op.tid, to_dev(k, w.heads.dtype), to_dev(v, w.heads.dtype), op.n_tokens)
                if dense is not None:
                    dense.append(op.tid, k, v)
            if led is not None:
                led.append(op.tid, op.n_tokens)
        elif op.kind == "fork":
            assert tuple(ap.apar_fork(h, op.tid, len(op.children))) == op.children
            if led is not None:
                assert tuple(led.fork(op.tid, len(op.children))) == op.children
            if dense is not None:
                assert tuple(dense.fork(op.tid, len(op.children))) == op.children
        elif op.kind == "free":
            ap.apar_free_thread(h, op.tid)
            if led is not None:
                led.free(op.tid)
            if dense is not None:
                dense.free(op.tid)
        if check_each and led is not None:
            books_equal(h, led)
    return live, live_nodes


def pool_for(w, num_blocks: int, dry_run: bool = False, **kw) -> "ap.Pool":
    hd = w.heads
    pool = ap.Pool(hd.n_q_heads, hd.n_kv_heads, hd.head_dim, hd.dtype, num_blocks, dry_run=dry_run, **kw)
    # every test pool verifies, before each launch that writes KV blocks, that no destination block is shared
    ap.apar_set_write_checks(pool.handle, True)
    return pool


def blocks_upper_bound(w) -> int:
    """Enough blocks for any replay of w: every node's segment rounded up, plus one copy per node."""
    return sum((n.seg_len + 15) // 16 + 1 for n in w.nodes) + 4


def nested_wide_tree(heads, seed=0):
    # a root with three children; two of them have more leaves below than one unit carries
    parents, lens = [-1, 0, 0, 0], [40, 20, 200, 33]
    for kid, n_leaves in ((1, 150), (2, 140), (3, 10)):
        for i in range(n_leaves):
            parents.append(kid)
            lens.append(1 + (i * 5) % 37)
    return manual_tree(parents, lens, heads, seed=seed, data_scale=0.5)


def random_forest(rng, n_roots, max_nodes):
    """Parents and segment lengths of a seeded random forest (deep and wide mixes, lengths around block boundaries)."""
    parents, segs = [], []
    for _ in range(n_roots):
        parents.append(-1)
        segs.append(int(rng.integers(1, 90)))
    while len(parents) < max_nodes:
        p = int(rng.integers(0, len(parents)))
        for _ in range(int(rng.integers(1, 7))):
            parents.append(p)
            segs.append(int(rng.choice([1, 2, 15, 16, 17, 31, 33, int(rng.integers(1, 70))])))
    return parents, segs


class PlanTablesOnDevice:
    """What the device's copy of the plan tables holds when a call that carries its plan over rewrites only the
    ints the library names as changed: follow() after every decode call keeps the copy the same way and compares
    it with the tables the library holds on the host (the ones the coverage check reads)."""

    def __init__(self, handle):
        self.handle = handle
        self.wgs = self.tiles = None
        self.carried = ap.apar_plan_counts(handle)[1]

    def follow(self) -> bool:
        h = self.handle
        wgs = np.array(ap.apar_last_plan_export(h, ap.APAR_PLAN_WORKGROUPS), dtype=np.int64)
        tiles = np.array(ap.apar_last_plan_export(h, ap.APAR_PLAN_TILES), dtype=np.int64)
        changed_w = np.array(ap.apar_last_plan_export(h, ap.APAR_PLAN_CHANGED_WORKGROUP_WORDS), dtype=np.int64)
        changed_t = np.array(ap.apar_last_plan_export(h, ap.APAR_PLAN_CHANGED_TILE_WORDS), dtype=np.int64)
        carried = ap.apar_plan_counts(h)[1]
        was_carried = carried > self.carried
        self.carried = carried
        if was_carried and self.wgs is not None:
            assert self.wgs.shape == wgs.shape and self.tiles.shape == tiles.shape, "a carried plan keeps its layout"
            self.wgs[changed_w] = wgs[changed_w]
            self.tiles[changed_t] = tiles[changed_t]
            assert np.array_equal(self.wgs, wgs), "workgroup ints changed that the library does not rewrite on the device"
            assert np.array_equal(self.tiles, tiles), "tile ints changed that the library does not rewrite on the device"
        else:
            assert was_carried or (len(changed_w) == 0 and len(changed_t) == 0)
            self.wgs, self.tiles = wgs, tiles
        return was_carried


def check_plan_covers_tables(handle, threads: Sequence[int], n_kv: int, rows_per_thread: int = 1) -> Dict[str, int]:
    """The exported plan must read, on behalf of every row group of every listed thread, exactly the
    blocks of that thread's table (each once, with the right fill counts); a thread is either written
    directly by the one unit that covers its whole path, or merged from exactly the partial results
    of the units that cover it."""
    wgs = np.array(ap.apar_last_plan_export(handle, ap.APAR_PLAN_WORKGROUPS), dtype=np.int64).reshape(-1, 32)
    tiles = np.array(ap.apar_last_plan_export(handle, ap.APAR_PLAN_TILES), dtype=np.int64).reshape(-1, 2)
    dfs = ap.apar_last_plan_export(handle, ap.APAR_PLAN_DFS_THREADS)
    path_ofs = ap.apar_last_plan_export(handle, ap.APAR_PLAN_PATH_OFS)
    path_ids = ap.apar_last_plan_export(handle, ap.APAR_PLAN_PATH_IDS)
    rpt, rps, n_sl = ap.apar_last_plan_export(handle, ap.APAR_PLAN_GEOMETRY)
    assert rpt == rows_per_thread and n_sl == -(-rpt // 16) and rps * n_sl >= rpt and rps <= 16
    cap = 16 // rps
    n = len(threads)
    assert sorted(dfs) == list(range(n)) and len(path_ofs) == n + 1
    seen = {}      # row group -> list of (block, valid)
    parts = {}     # rank -> set of partial rows
    direct = {}    # rank -> number of direct units
    tile_reads = 0
    for wg_index, wg in enumerate(wgs):
        coop_ofs, n_coop, grp_base, row_tiles, coop_full = wg[0], wg[1], wg[2], wg[3] & 255, wg[3] >> 8
        # 32 marks a matrix unit: a stand-alone chunk for up to 128 rows of whole threads, all named by entry 0
        assert row_tiles in (1, 2, 32)
        if wg_index:  # classes are stored matrix units, 2, 1
            assert row_tiles <= wgs[wg_index - 1][3] & 255
        if row_tiles == 32:
            assert wg[4 + 3] > 0 and (wg[4 + 3] // n_sl) * rpt <= 128 and wg[4 + 3] % n_sl == 0 and wg[4 + 2] % n_sl == 0
            assert wg[4 + 2] == grp_base and not wg[4 + 5] & 1 and wg[4 + 1] == 0
            assert all(wg[4 + 6 * k + 3] == 0 for k in (1, 2, 3))
            assert ((tiles[coop_ofs:coop_ofs + n_coop, 1] >> 10) & 1023 == wg[4 + 3]).all()
        # every list holds its full tiles first, then its open ones, and says how many are full
        assert 0 <= coop_full <= n_coop
        fills = (tiles[coop_ofs:coop_ofs + n_coop, 1] >> 20) & 31
        assert (fills[:coop_full] == 16).all() and (fills[coop_full:] < 16).all()
        tile_reads += n_coop
        for k in range(4):
            t_ofs, n_t, g_lo, n_g, pbase, flags = wg[4 + 6 * k: 10 + 6 * k]
            assert 0 <= n_g <= (128 if row_tiles == 32 else row_tiles * cap)
            fills = (tiles[t_ofs:t_ofs + n_t, 1] >> 20) & 31
            assert 0 <= wg[28 + k] <= n_t
            assert (fills[:wg[28 + k]] == 16).all() and (fills[wg[28 + k]:] < 16).all()
            tile_reads += n_t
            if n_g == 0:
                assert n_t == 0
                continue
            for g in range(g_lo, g_lo + n_g):
                rank = g // n_sl
                lst = seen.setdefault(g, [])
                for blk, meta in tiles[coop_ofs:coop_ofs + n_coop]:
                    lo, hi, valid = meta & 1023, (meta >> 10) & 1023, (meta >> 20) & 31
                    assert 1 <= valid <= 16 and lo < hi
                    if lo <= g - grp_base < hi:
                        lst.append((int(blk), int(valid)))
                for blk, meta in tiles[t_ofs:t_ofs + n_t]:
                    lo, hi, valid = meta & 1023, (meta >> 10) & 1023, (meta >> 20) & 31
                    assert 1 <= valid <= 16 and lo < hi <= n_g
                    if lo <= g - g_lo < hi:
                        lst.append((int(blk), int(valid)))
                if flags & 1:
                    direct.setdefault(rank, set()).add(wg_index)
                else:
                    parts.setdefault(rank, set()).add(int(pbase + rank - g_lo // n_sl))
    assert sorted(seen) == list(range(n * n_sl)), "every row group of every thread must be covered"
    all_parts = []
    for rank in range(n):
        i = dfs[rank]
        t = threads[i]
        table = ap.apar_thread_block_table(handle, t)
        L = ap.apar_thread_len(handle, t)
        for sl in range(n_sl):
            got = seen[rank * n_sl + sl]
            assert sorted(b for b, _ in got) == sorted(table), f"thread {t}: plan reads {got}, table is {table}"
            assert sum(v for _, v in got) == L
            assert all(v == 16 for b, v in got if b != table[-1])
        mine = set(path_ids[path_ofs[i]:path_ofs[i + 1]])
        if rank in direct:
            assert len(direct[rank]) == 1 and rank not in parts and not mine
        else:
            assert mine == parts[rank] and len(mine) == path_ofs[i + 1] - path_ofs[i]
            all_parts += list(mine)
    info = ap.apar_last_plan_info(handle)
    assert len(all_parts) == len(set(all_parts)), "a partial-result row belongs to one thread"
    assert info.n_partial_rows == len(all_parts)
    assert info.n_units == len(wgs) * n_kv
    uniq = set()
    for t in threads:
        uniq.update(ap.apar_thread_block_table(handle, t))
    assert info.unique_blocks == len(uniq)
    assert info.path_tokens == sum(ap.apar_thread_len(handle, t) for t in threads)
    return {"unit_block_reads": tile_reads, "unique_blocks": len(uniq), "partial_rows": len(all_parts),
            "direct_threads": len(direct)}


def check_prefill_plan(handle, threads: Sequence[int], m: Sequence[int], group: int) -> int:
    """The exported plan of a prefill call must show every query token exactly the token slots of its
    thread's table up to and including its own position, each once.  Returns the number of tile reads."""
    wgs = np.array(ap.apar_last_plan_export(handle, ap.APAR_PLAN_WORKGROUPS), dtype=np.int64).reshape(-1, 32)
    tiles = np.array(ap.apar_last_plan_export(handle, ap.APAR_PLAN_TILES), dtype=np.int64).reshape(-1, 2)
    rpt, rps, n_sl = ap.apar_last_plan_export(handle, ap.APAR_PLAN_GEOMETRY)
    assert (rpt, rps, n_sl) == (group, group, 1)
    cap = 16 // group
    seen = {}  # query token -> list of (block, slot)
    reads = 0

    def show(lst, blk, meta, ahead):
        fill = (meta >> 20) & 31
        limit = min(fill, ((meta >> 25) & 31) + ahead) if meta >> 30 else fill
        assert 1 <= fill <= 16 and limit >= 1
        lst += [(int(blk), s) for s in range(limit)]

    for wi, wg in enumerate(wgs):
        coop_ofs, n_coop, grp_base, row_tiles, coop_full = wg[0], wg[1], wg[2], wg[3] & 255, wg[3] >> 8
        assert row_tiles in (1, 2) and (wi == 0 or row_tiles <= wgs[wi - 1][3] & 255)
        reads += n_coop
        for k in range(4):
            t_ofs, n_t, g_lo, n_g, _, flags = wg[4 + 6 * k: 10 + 6 * k]
            assert 0 <= n_g <= row_tiles * cap
            if n_g == 0:
                assert n_t == 0
                continue
            assert flags & 1
            reads += n_t
            own = tiles[t_ofs:t_ofs + n_t]
            plain = [((mt >> 20) & 31) == 16 for mt in own[:, 1]]
            assert all(plain[:wg[28 + k]]) and not any(plain[wg[28 + k]:])
            for g in range(g_lo, g_lo + n_g):
                lst = seen.setdefault(int(g), [])
                for blk, meta in tiles[coop_ofs:coop_ofs + n_coop]:
                    lo, hi = meta & 1023, (meta >> 10) & 1023
                    assert ((meta >> 20) & 31) == 16 and not meta >> 30
                    if lo <= g - grp_base < hi:
                        show(lst, blk, meta, g - grp_base - lo)
                for blk, meta in own:
                    lo, hi = meta & 1023, (meta >> 10) & 1023
                    assert lo < hi <= n_g
                    if lo <= g - g_lo < hi:
                        show(lst, blk, meta, g - g_lo - lo)
    row = 0
    for t, mi in zip(threads, m):
        table = ap.apar_thread_block_table(handle, t)
        L = ap.apar_thread_len(handle, t)
        for r in range(mi):
            pos = L - mi + r
            want = [(table[x // 16], x % 16) for x in range(pos + 1)]
            assert sorted(seen[row]) == want, f"query token {row} (thread {t}, position {pos})"
            row += 1
    assert sorted(seen) == list(range(row))
    return reads
