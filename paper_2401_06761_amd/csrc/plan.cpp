// Plan builder: groups the listed threads by the blocks they share and lays the
// work out as workgroups of four wavefronts.
//
// Sharing only ever comes from forks, which hand a child the parent's whole table,
// and copy-on-write only replaces a tail.  Hence two tables that agree at one
// position agree at every earlier one, the set of live threads holding a table's
// block can only shrink along the table, and a maximal run of positions with one
// refcount is a run with one set of holders: a segment.  Every holder has the same
// run, so only the first listed holder walks it; the others find it by its first
// block and skip over it.  Segments form a forest (a segment's parent is the run
// before it in any holder's table); numbering the threads depth-first makes every
// segment's holders a contiguous range of ranks.
//
// Units.  Partial results are expensive: small writes mixed into the streaming
// reads cost far more than their size.  So a whole subtree of the forest is given
// to ONE unit whenever its query rows fit one workgroup (4 wavefronts x 16 or 32 rows;
// the fewest rows per wavefront that hold them are chosen):
// the rows' softmax state then stays in registers from the shared prefix down to
// each private tail, and threads whose entire path lies inside the unit get their
// output written directly.  Inside such a unit a block whose holders all sit in one
// wavefront goes on that wavefront's private list (no barrier, registers only);
// blocks needed by several wavefronts go on the shared list (staged once in LDS).
// A subtree with too many ROWS for one workgroup is cut by rank instead: its threads,
// in depth-first order, go to units of consecutive ranks, every unit full, and a unit
// reads every segment on the root paths of its threads - the segments near the root
// once per unit (as often as stand-alone units would read them), everything for its
// rows' state to stay in registers, nothing to merge afterwards.  Only where that does
// not work (partial results above, more blocks than a unit may be given, long segments
// with many rows that are better off on the matrix kernel) a top segment stands alone,
// chunked, with one partial result per (chunk, thread), and its children are tried
// again.  Attention is a set operation, so a unit may visit its blocks in any order.
#include "plan.hpp"

#include <algorithm>
#include <climits>

namespace apar {

void PlanHost::clear() {
    wgs.clear(), tiles.clear(), dfs_threads.clear(), path_ofs.clear(), path_ids.clear();
    segs.clear(), thread_last_seg.clear(), end_threads.clear(), order.clear(), stack.clear();
    path_len.clear(), narrow_items.clear(), wide_items.clear(), open_tmp.clear();
    n_partial_rows = n_segments = unique_blocks = unique_tokens = path_tokens = n_direct_threads = full_blocks = 0;
    any_partial = false;
    tails.clear(), tile_owner.clear(), spare.clear(), item_wg.clear(), item_slot.clear();
    dirty_wg_words.clear(), dirty_tile_words.clear();
    reusable = false;
    n_patched = 0;
}

namespace {

constexpr int B = kBlockTokens;

inline int32_t make_meta(int lo, int hi, int valid) { return lo | (hi << 10) | (valid << 20); }

struct Builder {
    PlanHost& ph;
    const PlanParams& prm;
    int n_sl, rps, cap;  // slices per thread, rows per slice, row groups per wavefront
    // per segment: first partial row it produces itself (stand-alone: n_chunks * n_shr rows; unit root
    // that is not direct: n_shr rows), and how many chunks
    std::vector<int32_t> part0, n_chunks;

    Builder(PlanHost& p, const PlanParams& q) : ph(p), prm(q) {
        n_sl = (q.rows_per_thread + 15) / 16;
        rps = (q.rows_per_thread + n_sl - 1) / n_sl;
        cap = 16 / rps;
    }

    // fewest 16-row tiles per wavefront with which one workgroup holds `groups` row groups (the most if none does)
    int pick_row_tiles(int groups) const {
        int nt = 1;
        while (nt < kMaxRowTiles && groups > 4 * nt * cap) nt *= 2;
        return nt;
    }

    // Pre-order walk of the subtree of `root`; f(segment index).
    template <class F>
    void for_subtree(int32_t root, F&& f) {
        std::vector<int32_t>& st = ph.stack;
        const size_t base = st.size();
        st.push_back(root);
        while (st.size() > base) {
            const int32_t s = st.back();
            st.pop_back();
            f(s);
            // children in reverse, so that the first child is visited first
            const size_t mark = st.size();
            for (int32_t c = ph.segs[s].first_child; c >= 0; c = ph.segs[c].next_sibling) st.push_back(c);
            std::reverse(st.begin() + mark, st.end());
        }
    }

    // Segment sg is the last of its one listed holder: remember which item's list (wide item and wavefront
    // 0..3 or kSharedList; kNarrowItem: the narrow item's only list) reads the thread's own last blocks, for
    // which row groups; build_plan turns the item into the workgroup it ends up in.
    static constexpr int32_t kNarrowItem = 8;
    static bool is_tail(const PlanHost::Segment& sg) { return sg.n_shr == 1 && sg.n_end == 1; }
    void note_tail(const PlanHost::Segment& sg, size_t item, int32_t slot, int lo, int hi) {
        PlanHost::Tail& t = ph.tails[ph.end_threads[sg.end_ofs]];
        t.wg = (int32_t)item;
        t.slot = slot;
        t.lohi = make_meta(lo, hi, 0);
    }
    void leave_slack(int n_tails) { ph.tiles.resize(ph.tiles.size() + (size_t)n_tails * PlanHost::kTailSlack); }
    void push_wide(PlanHost::WideItem& wi) {
        wi.id = (int32_t)ph.wide_items.size();
        ph.wide_items.push_back(wi);
    }

    void emit_narrow(int32_t tile_ofs, int32_t n_tiles, int32_t n_full, int32_t grp_lo, int32_t n_grp,
                     int32_t part_base, int32_t flags) {
        PlanHost::NarrowItem it;
        it.item = WaveItem{tile_ofs, n_tiles, grp_lo, n_grp, part_base, flags};
        it.cost = n_tiles;
        it.n_full = n_full;
        ph.narrow_items.push_back(it);
    }

    // Blocks [b0, b0 + nb) of segment s for row groups [lo, hi): full tiles go to `full`, the open one
    // (only a segment's last block can be) to `open`.
    void push_tiles(std::vector<TileRef>& full, std::vector<TileRef>& open, const PlanHost::Segment& s, int b0, int nb,
                    int lo, int hi) {
        const int32_t* blk = s.blocks;
        int n_plain = nb;
        if (b0 + nb == s.n_blk && s.last_valid < B) n_plain = nb - 1;
        const int32_t meta = make_meta(lo, hi, B);
        const size_t at = full.size();
        full.resize(at + n_plain);
        for (int b = 0; b < n_plain; ++b) full[at + b] = TileRef{blk[b0 + b], meta};
        if (n_plain < nb) open.push_back(TileRef{blk[b0 + nb - 1], make_meta(lo, hi, s.last_valid)});
    }

    // Segment sid stands alone: chunks of its blocks, one partial result per (chunk, thread).
    void emit_standalone(int32_t sid) {
        PlanHost::Segment& s = ph.segs[sid];
        const int groups = s.n_shr * n_sl;
        const int chunk = std::max(1, prm.max_unit_tiles);
        const int first_nb = std::min(s.n_blk, chunk);
        const int nch = 1 + (s.n_blk - first_nb + chunk - 1) / chunk;
        n_chunks[sid] = nch;
        part0[sid] = (int32_t)ph.n_partial_rows;
        ph.n_partial_rows += (int64_t)nch * s.n_shr;
        ph.any_partial = true;
        const int32_t grp0 = s.t_lo * n_sl;
        const bool tail_seg = is_tail(s);  // (one holder: every chunk is a single item)
        // the chunk's tiles for row groups [0, hi) of a list owner
        auto chunk_tiles = [&](int, int b0, int nb, int hi) {
            ph.open_tmp.clear();
            push_tiles(ph.tiles, ph.open_tmp, s, b0, nb, 0, hi);
        };
        for (int c = 0; c < nch; ++c) {
            const int b0 = c == 0 ? 0 : first_nb + (c - 1) * chunk, nb = c == 0 ? first_nb : std::min(chunk, s.n_blk - b0);
            const int32_t pbase = part0[sid] + c * s.n_shr;
            const bool tail_here = tail_seg && c == nch - 1;
            if (groups <= cap) {
                const int32_t ofs = (int32_t)ph.tiles.size();
                chunk_tiles(c, b0, nb, groups);
                const int32_t n_full = (int32_t)ph.tiles.size() - ofs;
                ph.tiles.insert(ph.tiles.end(), ph.open_tmp.begin(), ph.open_tmp.end());
                if (tail_here) note_tail(s, ph.narrow_items.size(), kNarrowItem, 0, groups);
                emit_narrow(ofs, (int32_t)ph.tiles.size() - ofs, n_full, grp0, groups, pbase, 0);
                if (tail_here) leave_slack(1);
            } else if (prm.matrix_min_rows > 0 && (int64_t)s.n_shr * prm.rows_per_thread >= prm.matrix_min_rows &&
                       s.n_blk >= prm.matrix_min_blocks) {
                // matrix units: whole threads, as evenly over the workgroups as they go
                const int per_wg = kMatrixUnitMaxRows / prm.rows_per_thread;  // >= 2: rows_per_thread <= 64
                const int n_wg = (s.n_shr + per_wg - 1) / per_wg;
                const int each = (s.n_shr + n_wg - 1) / n_wg;
                for (int t0 = 0; t0 < s.n_shr; t0 += each) {
                    const int nt = std::min(each, s.n_shr - t0);
                    PlanHost::WideItem wi{};
                    wi.wg.coop_ofs = (int32_t)ph.tiles.size();
                    wi.wg.grp_base = grp0 + t0 * n_sl;
                    chunk_tiles(c, b0, nb, nt * n_sl);
                    wi.wg.row_tiles = kMatrixUnitRows | (((int32_t)ph.tiles.size() - wi.wg.coop_ofs) << 8);
                    ph.tiles.insert(ph.tiles.end(), ph.open_tmp.begin(), ph.open_tmp.end());
                    wi.wg.n_coop = (int32_t)ph.tiles.size() - wi.wg.coop_ofs;
                    wi.wg.w[0] = WaveItem{0, 0, wi.wg.grp_base, nt * n_sl, pbase + t0, 0};
                    for (int k = 1; k < 4; ++k) wi.wg.w[k] = WaveItem{0, 0, 0, 0, -1, 0};
                    wi.cost = wi.wg.n_coop;
                    wi.family = -1;
                    if (tail_here) {
                        note_tail(s, ph.wide_items.size(), PlanHost::kSharedList, 0, nt * n_sl);
                        leave_slack(1);
                    }
                    push_wide(wi);
                }
            } else {
                const int nt = pick_row_tiles(groups), wcap = nt * cap;
                for (int g0 = 0; g0 < groups; g0 += 4 * wcap) {
                    const int gn = std::min(4 * wcap, groups - g0);
                    PlanHost::WideItem wi{};
                    wi.wg.row_tiles = nt;
                    wi.wg.coop_ofs = (int32_t)ph.tiles.size();
                    wi.wg.grp_base = grp0 + g0;
                    chunk_tiles(c, b0, nb, gn);
                    wi.wg.row_tiles |= ((int32_t)ph.tiles.size() - wi.wg.coop_ofs) << 8;
                    ph.tiles.insert(ph.tiles.end(), ph.open_tmp.begin(), ph.open_tmp.end());
                    wi.wg.n_coop = (int32_t)ph.tiles.size() - wi.wg.coop_ofs;
                    for (int k = 0; k < 4; ++k) {
                        const int lo = k * wcap, cnt = std::max(0, std::min(wcap, gn - lo));
                        wi.wg.w[k] = WaveItem{0, 0, grp0 + g0 + lo, cnt, pbase + (g0 + lo) / n_sl, 0};
                    }
                    wi.cost = 2 * wi.wg.n_coop * nt;
                    wi.family = -1;
                    if (tail_here) {
                        note_tail(s, ph.wide_items.size(), PlanHost::kSharedList, 0, gn);
                        leave_slack(1);
                    }
                    push_wide(wi);
                }
            }
        }
    }

    // A unit over the consecutive depth-first ranks [r_lo, r_lo + n_thr).  The rows' softmax state stays in
    // registers over everything the unit reads: either the whole subtree of `root` (whose threads are exactly
    // those ranks), or - root < 0 - every segment on the root paths of those threads, listed in range_segs (a
    // slice of a larger subtree cut by rank; `family` names that subtree's top segment).
    struct UnitSpec {
        int32_t root, r_lo, n_thr, family;
        bool direct;
    };
    std::vector<int32_t> range_segs;   // segments read by the rank-range unit being emitted
    std::vector<int32_t> seg_mark;     // per segment: last rank-range unit that listed it

    // f(segment index, lo, hi): the segments a unit reads, with the row groups (relative to the unit's first)
    // that hold them
    template <class F>
    void for_unit_segments(const UnitSpec& u, F&& f) {
        const int groups = u.n_thr * n_sl;
        auto clipped = [&](int32_t m) {
            const PlanHost::Segment& sg = ph.segs[m];
            const int lo = std::max(0, (sg.t_lo - u.r_lo) * n_sl);
            const int hi = std::min(groups, (sg.t_lo + sg.n_shr - u.r_lo) * n_sl);
            f(m, lo, hi);
        };
        if (u.root >= 0) for_subtree(u.root, clipped);
        else
            for (int32_t m : range_segs) clipped(m);
    }

    // Returns the unit's first partial-result row (-1 for a direct unit).
    int32_t emit_unit(const UnitSpec& u) {
        const int groups = u.n_thr * n_sl;
        int32_t pbase = -1;
        if (!u.direct) {
            pbase = (int32_t)ph.n_partial_rows;
            ph.n_partial_rows += u.n_thr;
            ph.any_partial = true;
        } else {
            ph.n_direct_threads += u.n_thr;
        }
        const int32_t flags = u.direct ? kWaveDirect : 0;
        const int32_t grp0 = u.r_lo * n_sl;
        if (groups <= cap) {
            const int32_t ofs = (int32_t)ph.tiles.size();
            ph.open_tmp.clear();
            int n_tails = 0;
            for_unit_segments(u, [&](int32_t m, int lo, int hi) {
                const PlanHost::Segment& sg = ph.segs[m];
                push_tiles(ph.tiles, ph.open_tmp, sg, 0, sg.n_blk, lo, hi);
                if (is_tail(sg)) {
                    note_tail(sg, ph.narrow_items.size(), kNarrowItem, lo, hi);
                    ++n_tails;
                }
            });
            const int32_t n_full = (int32_t)ph.tiles.size() - ofs;
            ph.tiles.insert(ph.tiles.end(), ph.open_tmp.begin(), ph.open_tmp.end());
            emit_narrow(ofs, (int32_t)ph.tiles.size() - ofs, n_full, grp0, groups, pbase, flags);
            leave_slack(n_tails);
            return pbase;
        }
        // several wavefronts: give each a contiguous range of row groups, keeping subtrees that fit
        // one wavefront whole where possible
        const int nt = pick_row_tiles(groups), wcap = nt * cap;
        int wave_lo[4] = {0, 0, 0, 0}, wave_n[4] = {0, 0, 0, 0};
        int cur = 0, fill = 0;
        bool overflow = false;
        auto atom = [&](int lo_rel, int cnt) {
            if (overflow) return;
            if (fill + cnt > wcap) {
                wave_n[cur] = fill;
                if (++cur >= 4) {
                    overflow = true;
                    return;
                }
                wave_lo[cur] = lo_rel;
                fill = 0;
            }
            fill += cnt;
        };
        auto thread_atoms = [&](int lo_rel) {  // one thread: whole if it fits a wavefront, else slice by slice
            if (n_sl <= wcap) atom(lo_rel, n_sl);
            else
                for (int sl = 0; sl < n_sl; ++sl) atom(lo_rel + sl, 1);
        };
        if (u.root < 0) overflow = true;  // a slice cut by rank is full: dense packing
        else {
            // a walk that stops descending where a subtree fits one wavefront
            std::vector<int32_t>& st = ph.stack;
            const size_t base = st.size();
            st.push_back(u.root);
            while (st.size() > base && !overflow) {
                const int32_t m = st.back();
                st.pop_back();
                const PlanHost::Segment& sg = ph.segs[m];
                const int lo = (sg.t_lo - u.r_lo) * n_sl, mg = sg.n_shr * n_sl;
                if (mg <= wcap) {
                    atom(lo, mg);
                    continue;
                }
                for (int e = 0; e < sg.n_end; ++e) thread_atoms(lo + e * n_sl);  // threads that end here come first in depth-first order
                const size_t mark = st.size();
                for (int32_t c = sg.first_child; c >= 0; c = ph.segs[c].next_sibling) st.push_back(c);
                std::reverse(st.begin() + mark, st.end());
            }
            st.resize(base);
        }
        if (!overflow) wave_n[cur] = fill;
        if (overflow) {  // dense packing always fits: groups <= 4 * wcap
            for (int k = 0; k < 4; ++k) {
                wave_lo[k] = k * wcap;
                wave_n[k] = std::max(0, std::min(wcap, groups - k * wcap));
            }
        }
        // first pass: who owns each segment the unit reads (a wavefront whose row groups contain all its
        // rows here, else the shared list), and how long the lists get; second pass: write the tiles in place
        int n_plain[5] = {0, 0, 0, 0, 0}, n_open[5] = {0, 0, 0, 0, 0};  // [0]: shared list, [1 + k]: wavefront k
        int n_tails[5] = {0, 0, 0, 0, 0};
        std::vector<int32_t>& visit = ph.order;
        visit.clear();
        for_unit_segments(u, [&](int32_t m, int lo, int hi) {
            const PlanHost::Segment& sg = ph.segs[m];
            int owner = -1;
            for (int k = 0; k < 4; ++k)
                if (wave_n[k] > 0 && lo >= wave_lo[k] && hi <= wave_lo[k] + wave_n[k]) owner = k;
            visit.push_back(m);
            visit.push_back(owner);
            visit.push_back(lo);
            visit.push_back(hi);
            const bool open = sg.last_valid < B;
            n_plain[owner + 1] += sg.n_blk - (open ? 1 : 0);
            n_open[owner + 1] += open ? 1 : 0;
            n_tails[owner + 1] += is_tail(sg) ? 1 : 0;
        });
        const size_t base = ph.tiles.size();
        size_t total = 0;
        TileRef *plain_at[5], *open_at[5];
        size_t list_ofs[5];
        for (int l = 0; l < 5; ++l) {
            list_ofs[l] = base + total;
            total += (size_t)n_plain[l] + n_open[l] + (size_t)n_tails[l] * PlanHost::kTailSlack;
        }
        ph.tiles.resize(base + total);
        for (int l = 0; l < 5; ++l) {
            plain_at[l] = ph.tiles.data() + list_ofs[l];
            open_at[l] = plain_at[l] + n_plain[l];
        }
        for (size_t i = 0; i < visit.size(); i += 4) {
            const PlanHost::Segment& sg = ph.segs[visit[i]];
            const int owner = visit[i + 1];
            const int rel = owner >= 0 ? wave_lo[owner] : 0;
            const int lo = visit[i + 2] - rel, hi = visit[i + 3] - rel;
            const bool open = sg.last_valid < B;
            const int np = sg.n_blk - (open ? 1 : 0);
            const int32_t meta = make_meta(lo, hi, B);
            TileRef* dst = plain_at[owner + 1];
            for (int b2 = 0; b2 < np; ++b2) dst[b2] = TileRef{sg.blocks[b2], meta};
            plain_at[owner + 1] += np;
            if (open) *open_at[owner + 1]++ = TileRef{sg.blocks[np], make_meta(lo, hi, sg.last_valid)};
            if (is_tail(sg)) note_tail(sg, ph.wide_items.size(), owner >= 0 ? owner : PlanHost::kSharedList, lo, hi);
        }
        PlanHost::WideItem wi{};
        wi.wg.coop_ofs = (int32_t)list_ofs[0];
        wi.wg.n_coop = n_plain[0] + n_open[0];
        wi.wg.grp_base = grp0;
        wi.wg.row_tiles = nt | (n_plain[0] << 8);
        int longest = 0;
        for (int k = 0; k < 4; ++k) {
            const int32_t cnt = n_plain[k + 1] + n_open[k + 1];
            wi.wg.w[k] = WaveItem{(int32_t)list_ofs[k + 1], cnt, grp0 + wave_lo[k], wave_n[k],
                                  u.direct ? -1 : pbase + wave_lo[k] / n_sl, flags};
            wi.wg.n_full[k] = n_plain[k + 1];
            longest = std::max(longest, (int)cnt);
        }
        wi.cost = nt * (2 * wi.wg.n_coop + longest);
        wi.family = u.family;
        push_wide(wi);
        return pbase;
    }

    // A whole sharing subtree as one unit.
    void emit_fused(int32_t rid) {
        PlanHost::Segment& r = ph.segs[rid];
        const bool direct = prm.allow_direct && r.n_above == 0;
        const int32_t pbase = emit_unit(UnitSpec{rid, r.t_lo, r.n_shr, -1, direct});
        if (!direct) part0[rid] = pbase;
    }

    // The segments on the root paths of the threads with ranks [r_lo, r_lo + n_thr) -> range_segs; returns their blocks.
    int64_t collect_range(int32_t r_lo, int32_t n_thr, int32_t stamp) {
        range_segs.clear();
        int64_t blocks = 0;
        for (int32_t rank = r_lo; rank < r_lo + n_thr; ++rank)
            for (int32_t m = ph.thread_last_seg[ph.dfs_threads[rank]]; m >= 0 && seg_mark[m] != stamp; m = ph.segs[m].parent) {
                seg_mark[m] = stamp;  // everything above a marked segment is marked too
                range_segs.push_back(m);
                blocks += ph.segs[m].n_blk;
            }
        return blocks;
    }

    // The subtree of segment rid has more query rows than one workgroup carries (and nothing above it leaves
    // partial results): its threads are cut by rank into the fewest units that hold them, evenly filled.  Every
    // unit is direct.  Returns false, with nothing emitted, if some unit would read more blocks than it may.
    int32_t next_stamp = 0;
    bool emit_by_rank(int32_t rid) {
        const PlanHost::Segment& r = ph.segs[rid];
        const int per_unit = std::max(1, 4 * kMaxRowTiles * cap / n_sl);  // threads
        const int n_units = (r.n_shr + per_unit - 1) / per_unit;
        const int64_t block_cap = (int64_t)4 * prm.max_unit_tiles;
        if (seg_mark.size() != ph.segs.size()) seg_mark.assign(ph.segs.size(), -1);
        auto slice = [&](int k, int32_t& lo, int32_t& cnt) {
            lo = r.t_lo + (int32_t)((int64_t)r.n_shr * k / n_units);
            cnt = r.t_lo + (int32_t)((int64_t)r.n_shr * (k + 1) / n_units) - lo;
        };
        if (r.tiles_sub > block_cap)  // (otherwise no slice can exceed the cap)
            for (int k = 0; k < n_units; ++k) {
                int32_t lo, cnt;
                slice(k, lo, cnt);
                if (collect_range(lo, cnt, next_stamp++) > block_cap) return false;
            }
        for (int k = 0; k < n_units; ++k) {
            int32_t lo, cnt;
            slice(k, lo, cnt);
            collect_range(lo, cnt, next_stamp++);
            emit_unit(UnitSpec{-1, lo, cnt, rid, true});
        }
        for_subtree(rid, [&](int32_t m) { ph.segs[m].unit = rid; });
        return true;
    }

};

}  // namespace

int build_plan(const PlanThreadView* threads, int n, const int32_t* refcount, int32_t* seg_of, const PlanParams& prm,
               PlanHost& ph) {
    ph.clear();
    if (prm.rows_per_thread < 1 || prm.rows_per_thread > 64) return APAR_ERR_UNSUPPORTED;
    Builder bld(ph, prm);
    std::vector<PlanHost::Segment>& segs = ph.segs;

    // 1. segments and their forest
    ph.thread_last_seg.resize(n);
    for (int i = 0; i < n; ++i) {
        // the walk below hops between a thread's table, the segment marks and the refcounts of its first
        // block, all cold: fetch them a few threads ahead
        if (i + 16 < n) __builtin_prefetch(threads[i + 16].table);
        if (i + 8 < n) {
            const int32_t b0 = threads[i + 8].table[0];
            __builtin_prefetch(seg_of + b0);
            __builtin_prefetch(refcount + b0);
        }
        const PlanThreadView& t = threads[i];
        ph.path_tokens += t.len;
        int pos = 0;
        int32_t prev = -1;
        while (pos < t.n_blocks) {
            const int32_t first = t.table[pos];
            int32_t sid = seg_of[first];
            if (sid < 0) {
                // refcounts never grow along a table (holders only drop out), so the run of equal
                // refcounts ends where a galloping search says it does
                const int32_t r = refcount[first];
                int end = pos + 1;
                if (end < t.n_blocks && refcount[t.table[end]] == r) {
                    int step = 1, good = end;  // table[good] is known to be in the run
                    while (good + step < t.n_blocks && refcount[t.table[good + step]] == r) {
                        good += step;
                        step *= 2;
                    }
                    int bad = std::min(good + step, (int)t.n_blocks);  // first position known to be outside (or the end)
                    while (bad - good > 1) {
                        const int mid = good + (bad - good) / 2;
                        if (refcount[t.table[mid]] == r) good = mid;
                        else bad = mid;
                    }
                    end = good + 1;
                }
                sid = (int32_t)segs.size();
                seg_of[first] = sid;
                PlanHost::Segment s{};
                s.blocks = t.table + pos;
                s.n_blk = end - pos;
                s.last_valid = (end == t.n_blocks) ? (int32_t)(t.len - (int64_t)(t.n_blocks - 1) * B) : B;
                s.parent = prev;
                s.first_child = s.last_child = s.next_sibling = -1;
                s.unit = -1;
                segs.push_back(s);
                if (prev >= 0) {
                    if (segs[prev].last_child >= 0) segs[segs[prev].last_child].next_sibling = sid;
                    else segs[prev].first_child = sid;
                    segs[prev].last_child = sid;
                }
            }
            segs[sid].n_shr += 1;
            prev = sid;
            pos += segs[sid].n_blk;
        }
        ph.thread_last_seg[i] = prev;
        segs[prev].n_end += 1;
    }
    for (const PlanHost::Segment& s : segs) seg_of[s.blocks[0]] = -1;  // scratch left clean
    const int32_t n_seg = (int32_t)segs.size();
    ph.n_segments = n_seg;

    // 2. threads that end at each segment, in listed order
    {
        int32_t acc = 0;
        for (PlanHost::Segment& s : segs) {
            s.end_ofs = acc;
            acc += s.n_end;
            s.n_end = 0;
        }
        ph.end_threads.resize(n);
        for (int i = 0; i < n; ++i) {
            PlanHost::Segment& s = segs[ph.thread_last_seg[i]];
            ph.end_threads[s.end_ofs + s.n_end++] = i;
        }
    }

    // 3. depth-first ranks; 4. subtree sizes
    ph.dfs_threads.resize(n);
    {
        int32_t rank = 0;
        for (int32_t r = 0; r < n_seg; ++r) {
            if (segs[r].parent >= 0) continue;
            bld.for_subtree(r, [&](int32_t m) {
                PlanHost::Segment& s = segs[m];
                s.t_lo = rank;
                for (int e = 0; e < s.n_end; ++e) ph.dfs_threads[rank++] = ph.end_threads[s.end_ofs + e];
            });
        }
        for (int32_t m = 0; m < n_seg; ++m) segs[m].tiles_sub = segs[m].n_blk;
        for (int32_t m = n_seg - 1; m >= 0; --m)  // children are created after their parents
            if (segs[m].parent >= 0) segs[segs[m].parent].tiles_sub += segs[m].tiles_sub;
    }

    // 5. cut the forest into units, parents first
    bld.part0.assign(n_seg, -1);
    bld.n_chunks.assign(n_seg, 0);
    bld.seg_mark.clear();
    {
        PlanHost::Tail none{};
        none.wg = none.slot = none.tile = -1;
        ph.tails.assign(n, none);
    }
    const int cap = bld.cap, n_sl = bld.n_sl;
    for (int32_t m = 0; m < n_seg; ++m) {
        PlanHost::Segment& s = segs[m];
        ph.unique_blocks += s.n_blk;
        ph.unique_tokens += (int64_t)(s.n_blk - 1) * B + s.last_valid;
        ph.full_blocks += s.n_blk - (s.last_valid < B ? 1 : 0);
        if (s.unit >= 0) continue;  // part of a subtree that was cut by rank
        const int32_t par = s.parent;
        if (par >= 0 && segs[par].unit >= 0) {
            s.unit = segs[par].unit;
            s.n_above = segs[par].n_above;
            continue;
        }
        s.n_above = par >= 0 ? segs[par].n_above + bld.n_chunks[par] : 0;
        const int groups = s.n_shr * n_sl;
        const bool few_rows = groups <= 4 * kMaxRowTiles * cap;
        if (prm.fuse && few_rows && s.tiles_sub <= (int64_t)(groups <= cap ? 1 : 4) * prm.max_unit_tiles) {
            s.unit = m;  // a unit is named after its root segment
            bld.emit_fused(m);
            continue;
        }
        // Too many rows (or blocks) below for one unit.  Too many ROWS: the subtree is cut by rank into full
        // units that each read the segments above their threads again (as often as stand-alone units would
        // read them) and write nothing but output rows; that needs the path above to be free of partial
        // results, so that the units are direct.  Long segments with many rows are better off alone on the
        // matrix kernel, and with too many blocks for few rows a segment is better read once: those stand
        // alone - chunked, one partial result per (chunk, thread), merged afterwards - and their children
        // are tried again.
        const bool to_matrix = prm.matrix_min_rows > 0 && (int64_t)s.n_shr * prm.rows_per_thread >= prm.matrix_min_rows &&
                               s.n_blk >= prm.matrix_min_blocks;
        if (prm.fuse && prm.inline_shared && prm.allow_direct && s.n_above == 0 && !to_matrix && !few_rows && bld.emit_by_rank(m))
            continue;
        bld.emit_standalone(m);
    }
    if (ph.n_partial_rows > INT32_MAX / 2 || ph.tiles.size() > (size_t)INT32_MAX / 2) return APAR_ERR_UNSUPPORTED;

    // 6. which partial results each listed thread has to merge
    ph.path_len.assign(n, 0);
    ph.path_ofs.assign(n + 1, 0);
    for (int pass = 0; pass < 2; ++pass) {
        for (int32_t rank = 0; rank < n; ++rank) {
            const int i = ph.dfs_threads[rank];
            int32_t cnt = 0;
            int32_t* dst = pass ? ph.path_ids.data() + ph.path_ofs[i] : nullptr;
            for (int32_t m = ph.thread_last_seg[i]; m >= 0; m = segs[m].parent) {
                const PlanHost::Segment& s = segs[m];
                if (s.unit >= 0) {
                    if (s.unit != m) continue;  // the unit's root accounts for the whole unit
                    if (bld.part0[m] >= 0) {
                        if (dst) dst[cnt] = bld.part0[m] + (rank - s.t_lo);
                        ++cnt;
                    }
                } else {
                    for (int c = 0; c < bld.n_chunks[m]; ++c) {
                        if (dst) dst[cnt] = bld.part0[m] + c * s.n_shr + (rank - s.t_lo);
                        ++cnt;
                    }
                }
            }
            if (!pass) ph.path_len[i] = cnt;
        }
        if (!pass) {
            for (int i = 0; i < n; ++i) ph.path_ofs[i + 1] = ph.path_ofs[i] + ph.path_len[i];
            ph.path_ids.resize(ph.path_ofs[n]);
        }
    }

    // 7. workgroups: matrix units, then by row tiles per wavefront (2, 1); within a class the heaviest first,
    // but the units cut out of one subtree stay together (ordered among the others by their heaviest)
    {
        std::vector<int32_t>& fam = ph.order;  // per segment: cost of the heaviest unit of the family it roots
        fam.assign(n_seg, 0);
        for (const PlanHost::WideItem& w : ph.wide_items)
            if (w.family >= 0) fam[w.family] = std::max(fam[w.family], w.cost);
        for (PlanHost::WideItem& w : ph.wide_items) w.family_cost = w.family >= 0 ? fam[w.family] : w.cost;
    }
    std::stable_sort(ph.wide_items.begin(), ph.wide_items.end(),
                     [](const PlanHost::WideItem& a, const PlanHost::WideItem& b) {
                         const int ta = a.wg.row_tiles & 255, tb = b.wg.row_tiles & 255;
                         if (ta != tb) return ta > tb;
                         if (a.family_cost != b.family_cost) return a.family_cost > b.family_cost;
                         if (a.family != b.family) return a.family > b.family;
                         return a.cost > b.cost;
                     });
    ph.wgs.reserve(ph.wide_items.size() + (ph.narrow_items.size() + 3) / 4);
    ph.n_wg_class[0] = ph.n_wg_class[1] = ph.n_wg_class[2] = 0;
    for (const PlanHost::WideItem& w : ph.wide_items) {
        ph.wgs.push_back(w.wg);
        ph.n_wg_class[(w.wg.row_tiles & 255) == kMatrixUnitRows ? 0 : (w.wg.row_tiles & 255) == 2 ? 1 : 2] += 1;
    }
    const size_t n_wide = ph.wgs.size();
    ph.item_wg.assign(ph.narrow_items.size(), -1);
    ph.item_slot.assign(ph.narrow_items.size(), -1);
    {
        // counting sort by cost, descending
        int32_t max_cost = 0;
        for (const PlanHost::NarrowItem& it : ph.narrow_items) max_cost = std::max(max_cost, it.cost);
        std::vector<int32_t>& cnt = ph.order;
        cnt.assign((size_t)max_cost + 2, 0);
        for (const PlanHost::NarrowItem& it : ph.narrow_items) cnt[max_cost - it.cost + 1] += 1;
        for (size_t c = 1; c < cnt.size(); ++c) cnt[c] += cnt[c - 1];
        std::vector<int32_t>& slot = ph.stack;
        slot.assign(ph.narrow_items.size(), 0);
        for (size_t k = 0; k < ph.narrow_items.size(); ++k) slot[cnt[max_cost - ph.narrow_items[k].cost]++] = (int32_t)k;
        // long units get a workgroup of their own and are split four ways; short ones are packed
        size_t k = 0;
        for (; k < slot.size() && ph.narrow_items[slot[k]].cost >= kSplitMinTiles; ++k) {
            const WaveItem& it = ph.narrow_items[slot[k]].item;
            const int32_t item_full = ph.narrow_items[slot[k]].n_full;
            WgDesc wg{};
            wg.grp_base = it.grp_lo;
            wg.row_tiles = 1;
            for (int j = 0; j < 4; ++j) {
                const int32_t b = (int32_t)((int64_t)it.n_tiles * j / 4), e = (int32_t)((int64_t)it.n_tiles * (j + 1) / 4);
                wg.w[j] = WaveItem{it.tile_ofs + b, e - b, it.grp_lo, it.n_grp, it.part_base, it.flags | kWaveSplit};
                wg.n_full[j] = std::max(0, std::min(e, item_full) - b);
            }
            // the item's open tiles, and the entries left free behind them, belong to the last quarter (if they all do)
            ph.item_wg[slot[k]] = (int32_t)ph.wgs.size();
            ph.item_slot[slot[k]] = item_full >= (int32_t)((int64_t)it.n_tiles * 3 / 4) ? 3 : -1;
            ph.wgs.push_back(wg);
        }
        for (; k < slot.size(); k += 4) {
            WgDesc wg{};
            for (int j = 0; j < 4; ++j) {
                if (k + j < slot.size()) {
                    wg.w[j] = ph.narrow_items[slot[k + j]].item;
                    wg.n_full[j] = ph.narrow_items[slot[k + j]].n_full;
                    ph.item_wg[slot[k + j]] = (int32_t)ph.wgs.size();
                    ph.item_slot[slot[k + j]] = j;
                } else {
                    wg.w[j] = WaveItem{0, 0, 0, 0, -1, 0};
                }
            }
            wg.grp_base = wg.w[0].grp_lo;
            wg.row_tiles = 1;
            ph.wgs.push_back(wg);
        }
    }
    ph.n_wg_class[2] += (int32_t)(ph.wgs.size() - n_wide);

    // 8. what patch_plan needs: each thread's table as the plan covers it, the list its own last blocks are on
    // (items have become workgroups by now), the tile of a last block that is still filling
    {
        std::vector<int32_t>& wide_pos = ph.order;  // order of emission -> workgroup
        wide_pos.assign(n_wide, 0);
        for (size_t k = 0; k < n_wide; ++k) wide_pos[ph.wide_items[k].id] = (int32_t)k;
        ph.tile_owner.assign(ph.tiles.size(), -1);
        ph.spare.assign(ph.wgs.size() * 5, 0);
        for (int i = 0; i < n; ++i) {
            PlanHost::Tail& t = ph.tails[i];
            const PlanThreadView& v = threads[i];
            t.len = v.len;
            t.n_blocks = v.n_blocks;
            t.tail_block = v.table[v.n_blocks - 1];
            t.tile = -1;
            if (t.slot == Builder::kNarrowItem) {
                const int32_t item = t.wg;
                t.wg = ph.item_wg[item];
                t.slot = ph.item_slot[item];
            } else if (t.slot >= 0) {
                t.wg = wide_pos[t.wg];
            }
            if (t.slot < 0) {
                t.wg = -1;
                continue;
            }
            ph.spare[(size_t)t.wg * 5 + t.slot] += PlanHost::kTailSlack;
            if (v.len - (int64_t)(v.n_blocks - 1) * B < B) {
                const WgDesc& wg = ph.wgs[t.wg];
                const bool shared = t.slot == PlanHost::kSharedList;
                const int32_t ofs = shared ? wg.coop_ofs : wg.w[t.slot].tile_ofs;
                const int32_t cnt = shared ? wg.n_coop : wg.w[t.slot].n_tiles;
                for (int32_t k = ofs + (shared ? wg.row_tiles >> 8 : wg.n_full[t.slot]); k < ofs + cnt; ++k)
                    if (ph.tiles[k].blk == t.tail_block) t.tile = k;
                if (t.tile < 0) t.wg = -1;
                else ph.tile_owner[t.tile] = i;
            }
        }
        ph.reusable = true;
    }
    return APAR_OK;
}

namespace {

struct ListView {
    int32_t ofs, n, n_full;
};
inline ListView list_of(const WgDesc& wg, int slot) {
    if (slot == PlanHost::kSharedList) return ListView{wg.coop_ofs, wg.n_coop, wg.row_tiles >> 8};
    return ListView{wg.w[slot].tile_ofs, wg.w[slot].n_tiles, wg.n_full[slot]};
}

}  // namespace

bool patch_plan(const PlanThreadView* threads, int n, bool no_copies, PlanHost& ph) {
    if (!ph.reusable || (size_t)n != ph.tails.size()) return false;
    ph.dirty_wg_words.clear(), ph.dirty_tile_words.clear();
    auto tile_changed = [&ph](int32_t idx, bool block_too = true) {
        if (block_too) ph.dirty_tile_words.push_back(2 * idx);
        ph.dirty_tile_words.push_back(2 * idx + 1);
    };
    // (the word a list's length or its count of full tiles is kept in: see WgDesc)
    auto count_changed = [&ph](int32_t wg, int slot, bool n_full) {
        const int word = slot == PlanHost::kSharedList ? (n_full ? 3 : 1) : (n_full ? 28 + slot : 4 + 6 * slot + 1);
        ph.dirty_wg_words.push_back(wg * 32 + word);
    };
    auto give_up = [&ph] {
        ph.reusable = false;
        return false;
    };
    // The tile at `idx` of a list now reads a full block: it changes places with the list's first open tile.
    auto to_full_part = [&](int32_t wg_index, int slot, int32_t idx) {
        WgDesc& wg = ph.wgs[wg_index];
        const ListView l = list_of(wg, slot);
        const int32_t f = l.ofs + l.n_full;
        if (f != idx) {
            std::swap(ph.tiles[f], ph.tiles[idx]);
            std::swap(ph.tile_owner[f], ph.tile_owner[idx]);
            if (ph.tile_owner[idx] >= 0) ph.tails[ph.tile_owner[idx]].tile = idx;
            tile_changed(f);
            tile_changed(idx);
        }
        ph.tile_owner[f] = -1;
        if (slot == PlanHost::kSharedList) wg.row_tiles += 1 << 8;
        else wg.n_full[slot] += 1;
        count_changed(wg_index, slot, true);
        ph.full_blocks += 1;
    };
    for (int i = 0; i < n; ++i) {
        if (i + 8 < n) {
            const PlanHost::Tail& ahead = ph.tails[i + 8];
            if (!no_copies) __builtin_prefetch(threads[i + 8].table + std::min(ahead.n_blocks, threads[i + 8].n_blocks) - 1);
            if (ahead.tile >= 0) __builtin_prefetch(&ph.tiles[ahead.tile], 1);
            else if (ahead.wg >= 0) __builtin_prefetch(&ph.wgs[ahead.wg], 1);  // a full last block: the next row opens a new one
        }
        PlanHost::Tail& t = ph.tails[i];
        const PlanThreadView& v = threads[i];
        if (v.n_blocks < t.n_blocks || v.len < t.len) return give_up();
        // (without a copy-on-write copy anywhere since, the block is the one it was)
        const int32_t at_tail = no_copies ? t.tail_block : v.table[t.n_blocks - 1];
        if (v.len == t.len) {
            if (v.n_blocks != t.n_blocks || at_tail != t.tail_block) return give_up();
            continue;
        }
        const int dn = v.n_blocks - t.n_blocks;
        if (t.wg < 0 || dn > 1) return give_up();
        WgDesc& wg = ph.wgs[t.wg];
        if (t.len - (int64_t)(t.n_blocks - 1) * B < B) {
            // the block that was filling: more rows, perhaps in its copy-on-write copy, perhaps full now
            if (t.tile < 0) return give_up();
            const int now = dn ? B : (int)(v.len - (int64_t)(v.n_blocks - 1) * B);
            ph.tiles[t.tile] = TileRef{at_tail, t.lohi | (now << 20)};
            tile_changed(t.tile, at_tail != t.tail_block);
            if (now == B) {
                to_full_part(t.wg, t.slot, t.tile);
                t.tile = -1;
            }
        } else if (dn == 0 || at_tail != t.tail_block) {
            return give_up();  // (a full last block stays as it is)
        }
        if (dn) {
            int32_t& left = ph.spare[(size_t)t.wg * 5 + t.slot];
            if (left <= 0) return give_up();
            left -= 1;
            const ListView l = list_of(wg, t.slot);
            const int32_t idx = l.ofs + l.n;
            const int now = (int)(v.len - (int64_t)(v.n_blocks - 1) * B);
            ph.tiles[idx] = TileRef{v.table[v.n_blocks - 1], t.lohi | (now << 20)};
            ph.tile_owner[idx] = i;
            tile_changed(idx);
            if (t.slot == PlanHost::kSharedList) wg.n_coop += 1;
            else wg.w[t.slot].n_tiles += 1;
            count_changed(t.wg, t.slot, false);
            t.tile = idx;
            ph.unique_blocks += 1;
            if (now == B) {
                to_full_part(t.wg, t.slot, idx);
                t.tile = -1;
            }
        }
        ph.unique_tokens += v.len - t.len;
        ph.path_tokens += v.len - t.len;
        t.len = v.len;
        t.n_blocks = v.n_blocks;
        t.tail_block = v.table[v.n_blocks - 1];
    }
    ph.n_patched += 1;
    return true;
}

int build_prefill_plan(const PrefillThreadView* threads, int n, int group, PlanHost& ph) {
    ph.clear();
    if (group < 1 || group > 16 || 16 % group != 0) return APAR_ERR_UNSUPPORTED;
    const int cap = 16 / group;  // query tokens per 16-row tile
    for (int i = 0; i < n; ++i) {
        const PrefillThreadView& t = threads[i];
        const int64_t L = t.len;
        for (int64_t r0 = 0; r0 < t.m;) {
            const int64_t left = t.m - r0;
            const int nt = left <= 4 * cap ? 1 : kMaxRowTiles;
            const int chunk = (int)std::min<int64_t>(left, 4 * nt * cap);
            const int W = (chunk + 3) / 4;            // tokens per wavefront (<= nt * cap)
            const int64_t p0 = L - t.m + r0;          // position of the workgroup's first query token
            const int n_sh = (int)((p0 + 1) / kBlockTokens);  // blocks wholly at or below that position: full
            PlanHost::WideItem wi{};
            wi.wg.coop_ofs = (int32_t)ph.tiles.size();
            wi.wg.n_coop = n_sh;
            wi.wg.grp_base = (int32_t)(t.q_base + r0);
            wi.wg.row_tiles = nt | (n_sh << 8);
            {
                const size_t at = ph.tiles.size();
                ph.tiles.resize(at + n_sh);
                const int32_t meta = make_meta(0, chunk, B);
                for (int b = 0; b < n_sh; ++b) ph.tiles[at + b] = TileRef{t.table[b], meta};
            }
            int longest = 0;
            for (int k = 0; k < 4; ++k) {
                const int w0 = k * W, cnt = std::max(0, std::min(W, chunk - w0));
                if (cnt == 0) {
                    wi.wg.w[k] = WaveItem{0, 0, wi.wg.grp_base, 0, -1, 0};
                    continue;
                }
                const int64_t pw0 = p0 + w0, p_last = pw0 + cnt - 1;
                const int32_t ofs = (int32_t)ph.tiles.size();
                int n_plain = 0;
                for (int64_t b = n_sh; b <= p_last / kBlockTokens; ++b) {
                    const int lo = (int)std::max<int64_t>(0, b * kBlockTokens - pw0);  // first token that sees slot 0
                    const int fill = (int)std::min<int64_t>(kBlockTokens, L - b * kBlockTokens);
                    const int64_t first = pw0 + lo - b * kBlockTokens + 1;             // slots that token sees
                    int32_t meta = make_meta(lo, cnt, fill);
                    if (first < fill) meta |= ((int32_t)first << 25) | (1 << 30);      // causal
                    if (fill == kBlockTokens) ++n_plain;  // (only a thread's last block can be open: full ones come first)
                    ph.tiles.push_back(TileRef{t.table[b], meta});
                }
                const int32_t n_tiles = (int32_t)ph.tiles.size() - ofs;
                wi.wg.w[k] = WaveItem{ofs, n_tiles, wi.wg.grp_base + w0, cnt, -1, kWaveDirect};
                wi.wg.n_full[k] = n_plain;
                longest = std::max(longest, (int)n_tiles);
            }
            wi.cost = nt * (2 * n_sh + longest);
            ph.wide_items.push_back(wi);
            r0 += chunk;
        }
    }
    if (ph.tiles.size() > (size_t)INT32_MAX / 2) return APAR_ERR_UNSUPPORTED;
    std::stable_sort(ph.wide_items.begin(), ph.wide_items.end(),
                     [](const PlanHost::WideItem& a, const PlanHost::WideItem& b) {
                         const int ta = a.wg.row_tiles & 255, tb = b.wg.row_tiles & 255;
                         return ta != tb ? ta > tb : a.cost > b.cost;
                     });
    ph.n_wg_class[0] = ph.n_wg_class[1] = ph.n_wg_class[2] = 0;
    ph.wgs.reserve(ph.wide_items.size());
    for (const PlanHost::WideItem& w : ph.wide_items) {
        ph.wgs.push_back(w.wg);
        ph.n_wg_class[(w.wg.row_tiles & 255) == kMatrixUnitRows ? 0 : (w.wg.row_tiles & 255) == 2 ? 1 : 2] += 1;
    }
    return APAR_OK;
}

}  // namespace apar
