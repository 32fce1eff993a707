// The decode plan: which workgroup reads which blocks on behalf of which threads.
// Host-only; the device-side layouts it fills are declared in apar_internal.hpp.
#pragma once

#include <cstdint>
#include <vector>

#include "apar_internal.hpp"

namespace apar {

struct PlanThreadView {  // what the planner needs to know about one listed thread
    const int32_t* table;
    int32_t n_blocks;
    int64_t len;
};

struct PlanHost {
    // device-format tables
    std::vector<WgDesc> wgs;            // by class (matrix units, then 2 and 1 row tiles per wavefront), heaviest first within a class
    int32_t n_wg_class[3] = {0, 0, 0};
    std::vector<TileRef> tiles;
    std::vector<int32_t> dfs_threads;   // listed-thread indices in depth-first order of the sharing tree
    std::vector<int32_t> path_ofs, path_ids;
    // totals
    int64_t n_partial_rows = 0, n_segments = 0, unique_blocks = 0, unique_tokens = 0, path_tokens = 0;
    int64_t full_blocks = 0;            // of the unique blocks, those with all sixteen slots filled
    int64_t n_direct_threads = 0;
    bool any_partial = false;

    // scratch kept between calls so that steady-state planning does not allocate
    struct Segment {
        const int32_t* blocks;    // the run inside the table of the first listed holder (tables outlive the plan build)
        int32_t n_blk, last_valid, n_shr;
        int32_t parent, first_child, last_child, next_sibling;
        int32_t n_end, end_ofs;   // listed threads whose table ends with this segment
        int32_t t_lo;             // depth-first rank of its first thread
        int32_t tiles_sub;        // blocks in its whole subtree
        int32_t unit;             // fused unit it belongs to, -1 if it stands alone
        int32_t n_above;          // partial results produced above it on the path (same for all its threads)
    };
    std::vector<Segment> segs;
    std::vector<int32_t> thread_last_seg, end_threads, order, stack;
    std::vector<int32_t> path_len;
    std::vector<TileRef> open_tmp;
    struct NarrowItem {
        WaveItem item;
        int32_t cost;
        int32_t n_full;  // full tiles at the head of the item's list
    };
    std::vector<NarrowItem> narrow_items;
    struct WideItem {
        WgDesc wg;
        int32_t cost;
        int32_t id;          // position in the order of emission
        int32_t family;      // top segment of the subtree the unit was cut out of by rank (-1: none): units of one family
                             // are launched next to each other, so that the segments they all read are found in L2
        int32_t family_cost; // cost of the family's heaviest unit (its own cost if it has no family)
    };
    std::vector<WideItem> wide_items;

    // What the next call needs to carry this plan over instead of building another (patch_plan): of every
    // listed thread, the table the plan covers and where the tile of its last block sits.
    struct Tail {
        int64_t len;         // the thread's length when the plan was made or last patched
        int32_t n_blocks;    // its table's length then
        int32_t tail_block;  // table[n_blocks - 1]
        int32_t tile;        // index in `tiles` of that block's tile while the block is filling, -1 once it is full
        int32_t wg, slot;    // the list its own last blocks are on: workgroup, and wavefront 0..3 or kSharedList;
                             // wg < 0: not known (the thread's last segment has another listed holder, or the list is
                             // one that cannot be grown in place)
        int32_t lohi;        // row groups of its tiles relative to that list's owner: lo | hi << 10
    };
    static constexpr int32_t kSharedList = 4;
    static constexpr int32_t kTailSlack = 4;  // unused tile entries left behind a list per thread whose tail is on it
    std::vector<Tail> tails;
    std::vector<int32_t> tile_owner;   // per entry of `tiles`: the listed thread whose filling last block it reads, else -1
    std::vector<int32_t> spare;        // per (workgroup, list): unused tile entries behind the list
    std::vector<int32_t> item_wg, item_slot;  // build scratch: where each narrow item / wide item ended up
    // what the last patch_plan changed, for a copy of the tables that is brought up to date instead of
    // written again: indices of 32-bit words of `wgs` and of `tiles` (a word may be listed twice)
    std::vector<int32_t> dirty_wg_words, dirty_tile_words;
    bool reusable = false;             // tails, tile_owner and spare describe wgs and tiles as they stand
    int32_t n_patched = 0;             // calls that carried this plan over since it was built

    void clear();
};

struct PlanParams {
    int32_t rows_per_thread;  // candidates * q heads per kv head
    int32_t max_unit_tiles;   // longest tile list one wavefront may be given
    bool allow_direct;        // threads whose whole path is one unit may write their output directly
    bool fuse;                // build tree-fused units (false: every segment stands alone)
    bool inline_shared = true;  // a subtree with more rows than one unit carries is cut by rank into direct units that each
                                // read the shared segments above their threads, instead of standing alone with partial results
    int32_t matrix_min_rows = 0;    // stand-alone segments with at least this many query rows (0: never) ...
    int32_t matrix_min_blocks = 0;  // ... and at least this many blocks become matrix units
};

struct PrefillThreadView {  // one listed thread of a prefill call
    const int32_t* table;
    int32_t n_blocks;
    int64_t len;
    int32_t m;        // its last m rows are the query tokens
    int64_t q_base;   // index of its first query token among all query tokens of the call
};

// Plan of a prefill call: the query tokens take the place of the listed threads of a decode plan (row
// group = query token, numbered across the call), a workgroup holds up to 128 / group consecutive tokens
// of one thread, the tiles below its first token go on its shared list and the tiles on the diagonal
// on the wavefronts' own lists, marked causal.  group = q heads per kv head, a divisor of 16.
int build_prefill_plan(const PrefillThreadView* threads, int n, int group, PlanHost& ph);

// seg_of: pool-sized scratch, all -1 on entry and on exit.  refcount: the pool's refcounts.
// Returns 0, or a negative apar_status.
int build_plan(const PlanThreadView* threads, int n, const int32_t* refcount, int32_t* seg_of, const PlanParams& prm,
               PlanHost& ph);

// Carries the plan in `ph` over to a call that lists, position by position, the same threads as the call it
// was built (or last patched) for - or threads forked from them since - with the same parameters; the caller
// vouches for that.  Tables only ever change from their last block on, so all there is to do is to follow
// each thread's tail: new fill counts, a last block replaced by its copy-on-write copy, a block that filled
// up and moves to the full part of its list, one new block put in an entry left free behind the list.
// Returns false - and the plan must then be built afresh - when a thread changed in any other way (its
// last segment has several listed holders, more than one new block, no entry left).  The totals in `ph`
// follow; its segment records do not (they describe the plan as it was built).
// no_copies: the caller knows that no block was replaced by a copy-on-write copy since that call, so that a
// table that has not grown need not be looked at.
bool patch_plan(const PlanThreadView* threads, int n, bool no_copies, PlanHost& ph);

}  // namespace apar
