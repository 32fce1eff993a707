// Internal declarations shared by the host side and the kernels of libapar.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apar.h"

namespace apar {

constexpr int kBlockTokens = 16;
constexpr int32_t kCodeSealed = 1 << 30;  // flag on a (block * 16 + slot) code: the block is sealed
constexpr int64_t kMaxPoolBlocks = (int64_t)1 << 26;  // block * 16 + slot must stay below the flag bit
static_assert(kMaxPoolBlocks * kBlockTokens <= kCodeSealed, "a slot code must not reach the sealed flag");

// ---------------------------------------------------------------------------
// Pool layout in HBM.
//
// The pool is [block][kv_head] tiles; a tile holds the K rows and then the V
// rows of the block's 16 token slots for that head.
//
// f32 pools: both halves are row-major [16][d].
//
// bf16 pools (d = 128; tile = 4 KiB of K + 4 KiB of V).  A block that is still
// filling (fewer than 16 slots written) is row-major too, so that appending a row
// is a few full-line writes.  When its sixteenth slot is written the block is
// SEALED: both halves are rewritten in the order the 16x16 matrix-core
// instructions consume them, so that a wavefront fills its operand registers with
// four fully coalesced 1 KiB loads per half and no shuffle or LDS pass.  Full
// blocks are never written again, and every thread that holds a block agrees on
// its fill count, so "filled slots < 16" is all a reader needs to know the format.
// Sealed layout, with lane = 16*g + c (g = 0..3, c = 0..15) and load index
// r = 0..3: the 16 bytes at  r*1024 + lane*16  hold
//   K half: K[token c][dims 32*g + 8*r .. +8]               (A operand of K.Q^T)
//   V half: V[tokens 4*g .. 4*g+3][dim 32*r + c] followed by
//           V[tokens 4*g .. 4*g+3][dim 32*r + 16 + c]       (A operand of V^T.P^T)
//
// fp8 pools (APAR_BF16_FP8KV) seal a block into fp8 codes (OCP e4m3) in the same element order, one
// byte per element: the K half is bytes [0, 2048) of the tile, the V half [2048, 4096), and piece r
// of a lane is the 8 bytes at  half + (r/2)*1024 + lane*16 + (r%2)*8  (a 16-byte load brings two
// pieces).  Bytes [4096, 4104) hold two floats, the scale of the K half and of the V half: powers
// of two, value = code * scale.  The rest of the 8 KiB tile is unused while the block is sealed.
// ---------------------------------------------------------------------------
constexpr int kFp8HalfBytes = 2048;   // one half (K or V) of a sealed fp8 tile
constexpr int kFp8ScaleOfs = 4096;    // float K scale, float V scale
__host__ __device__ inline int fp8_k_offset(int token, int dim) {  // byte offset of an element inside the K half
    const int r = (dim & 31) >> 3, lane = (dim >> 5) * 16 + token;
    return (r >> 1) * 1024 + lane * 16 + (r & 1) * 8 + (dim & 7);
}
__host__ __device__ inline int fp8_v_offset(int token, int dim) {  // byte offset of an element inside the V half
    const int r = dim >> 5, lane = (token >> 2) * 16 + (dim & 15);
    return (r >> 1) * 1024 + lane * 16 + (r & 1) * 8 + ((dim >> 4) & 1) * 4 + (token & 3);
}
__host__ __device__ inline int bf16_k_offset(int token, int dim) {  // byte offset inside the K half
    return ((dim & 31) >> 3) * 1024 + (((dim >> 5) * 16 + token) * 16) + (dim & 7) * 2;
}
__host__ __device__ inline int bf16_v_offset(int token, int dim) {  // byte offset inside the V half
    return (dim >> 5) * 1024 + (((token >> 2) * 16 + (dim & 15)) * 16) + ((dim >> 4) & 1) * 8 + (token & 3) * 2;
}

// ---------------------------------------------------------------------------
// Plan tables (built on the host, read by the attention and merge kernels).
//
// The listed threads are numbered in depth-first order of their sharing tree, so
// the threads that hold any given block are a contiguous range of ranks.  A
// thread's query rows (candidates x q heads of one kv group) are cut into
// `n_slices` slices of at most 16 rows; (thread, slice) is a "row group" with
// index rank * n_slices + slice.  A wavefront holds up to row_tiles * (16 / rows_per_slice)
// consecutive row groups as the columns of its row_tiles 16x16 tiles (a row group
// never straddles two tiles: group j of the wavefront sits in tile j / (16 / rows_per_slice)).
// ---------------------------------------------------------------------------
struct TileRef {     // one block to read, and the row groups it applies to
    int32_t blk;
    int32_t meta;    // lo | hi << 10 | valid << 20: row groups [lo, hi) relative to the list owner's first
                     // row group (the workgroup's for shared lists, the wavefront's for its own list);
                     // valid = filled token slots (1..16).  Bit 30 marks a causal tile (prefill): row
                     // group lo sees only the first `first` slots (bits 25-29, 1..16), group lo + 1 one
                     // more, and so on up to valid.
};

// Most 16-row tiles one wavefront is given.  The kernels take 4 as well, but with 64 rows of state a
// wavefront runs out of the 256 architectural registers and the compiler shuttles accumulators to and
// from the accumulation registers around every use: measured slower than two tiles plus partial results
// (decode) or more workgroups (prefill), so the plans stop at 2.
constexpr int kMaxRowTiles = 2;
// Value of a workgroup descriptor's row-tile byte that marks a matrix unit (bf16 pools): a stand-alone
// chunk of a shared segment for up to 128 query rows, run by the 32x32 kernel.  Its shared tile list is
// the chunk; wavefront entry 0 names the threads (row groups of whole threads, rows laid flat over the
// workgroup) and the first thread's partial-result row; entries 1..3 are empty.
constexpr int kMatrixUnitRows = 32;
constexpr int kMatrixUnitMaxRows = 128;

struct WaveItem {    // what one wavefront computes
    int32_t tile_ofs, n_tiles;  // its own tile list
    int32_t grp_lo, n_grp;      // its row groups [grp_lo, grp_lo + n_grp); n_grp == 0: nothing to compute
    int32_t part_base;          // partial-result row of the thread that owns row group grp_lo
    int32_t flags;              // kWaveDirect: normalise and write the output rows instead of partial results
};
constexpr int32_t kWaveDirect = 1;
constexpr int32_t kWaveSplit = 2;  // the group's four wavefronts hold the SAME rows and a quarter of the tiles each;
                                   // their results are combined in LDS and wavefront 0 writes them
constexpr int kSplitMinTiles = 16; // shorter private units are packed four to a workgroup instead

// Every tile list holds its full tiles (16 filled slots) first and its open ones last, so that
// the kernels can run the bulk of a list through a loop that knows nothing of open tiles.
struct WgDesc {      // one 256-thread workgroup: a shared tile list, then one private list per wavefront
    int32_t coop_ofs, n_coop;   // tiles every wavefront of the group sees (staged once through LDS)
    int32_t grp_base;           // row group that the shared list's ranges are relative to
    int32_t row_tiles;          // bits 0-7: 16-row tiles per wavefront (1 or 2; the f32 kernel also takes 4);
                                // bits 8-31: full shared tiles
    WaveItem w[4];
    int32_t n_full[4];          // full tiles at the head of each wavefront's own list
};
static_assert(sizeof(WgDesc) == 128, "WgDesc is read with aligned scalar loads");

struct PlanDev {              // device pointers of one staged plan
    const WgDesc* wgs;
    const TileRef* tiles;
    const int32_t* dfs_threads;  // rank -> index into the listed threads (null: the identity)
    const int32_t* path_ofs;     // [n_threads + 1], by listed index
    const int32_t* path_ids;     // partial-result rows to merge for each listed thread (none: written directly)
    int32_t n_wg;
    int32_t n_wg_class[3];       // matrix units, workgroups with 2 and with 1 row tiles per wavefront, stored in that order
    int32_t n_threads;
    int32_t rows_per_thread, rows_per_slice, n_slices;
};

struct PrefillWg {            // one workgroup of the bf16 prefill kernel: consecutive query tokens of one thread
    int32_t table_ofs;        // the thread's block table inside the staged tables
    int32_t q_row0;           // index of its first query token among the call's query tokens
    int32_t p0;               // position of that token in the thread
    int32_t n_tok;            // query tokens it holds (n_tok * group <= 128 rows)
    int32_t len;              // the thread's length
    int32_t pad[3];
};
static_assert(sizeof(PrefillWg) == 32, "PrefillWg is read with one aligned scalar load");

struct Shape {
    int32_t n_q, n_kv, d, group;  // group = n_q / n_kv
    int32_t dtype;                // element type of rows at the interface and in blocks that are still filling: APAR_F32 or APAR_BF16
    int32_t fp8_sealed;           // 1: full blocks are kept in fp8 with a power-of-two scale per (block, kv head) and half
    float scale_log2e;            // softmax scale * log2(e): logits are kept in base 2
    int64_t tile_bytes;           // one (block, kv head): 2 * 16 * d * e
    int64_t block_bytes;          // n_kv tiles
};

// Partial results: for partial row p, candidate c, q head h the slot is
// (p * n_cand + c) * n_q + h; part_o holds d floats per slot, part_ml two (max, sum).
struct PartialBuf {
    float* o;
    float* ml;
};

// Side streams on which the attention kernels of different row-tile classes run next to each
// other (each class alone would leave most of the chip idle during its tail).  Created on first
// use by the launcher, released by the pool; all at the default priority.
struct ClassStreams {
    hipStream_t aux[2] = {nullptr, nullptr};
    hipEvent_t fork = nullptr, join[2] = {nullptr, nullptr};
    bool serial = false;  // true: every class is launched on the caller's stream, one after the other, and
                          // no stream or event is ever created (for the entry point that must not allocate)
};

// Where `device`'s copy of the library's static workspace (APAR_FIXED_PLAN_BYTES of plan tables followed by
// APAR_FIXED_PARTIAL_BYTES of partial results) lives.  `device` must be the current device.  The address is
// asked for once per device and kept.
hipError_t fixed_workspace_of_device(int device, char** out);

// ---- launchers (defined next to their kernels) ------------------------------
hipError_t launch_append_rows(const Shape& s, void* pool, const void* k, const void* v, const int32_t* dst_codes,
                              const int32_t* src_rows, int n_rows, hipStream_t st);
hipError_t launch_block_copies(const Shape& s, void* pool, const int32_t* src_dst_pairs, int n_pairs,
                               hipStream_t st);
hipError_t launch_seal_blocks(const Shape& s, void* pool, const int32_t* blocks, int n_blocks, hipStream_t st);
// words[pairs[2 i]] = pairs[2 i + 1] for i < n_pairs (device pointers; `pairs` 8-byte aligned)
hipError_t launch_scatter_words(int32_t* words, const int32_t* pairs, int n_pairs, hipStream_t st);
hipError_t launch_read_rows(const Shape& s, const void* pool, const int32_t* src_codes, int n_rows, void* k_out,
                            void* v_out, hipStream_t st);
hipError_t launch_attention_partial(const Shape& s, const void* pool, const void* q, const PlanDev& plan, int n_cand,
                                    PartialBuf part, const void* cand_k, const void* cand_v, const uint8_t* mask,
                                    void* out, ClassStreams& cs, hipStream_t st);
hipError_t launch_prefill_bf16(const Shape& s, const void* pool, const void* q, const PrefillWg* wgs,
                               const int32_t* tables, int n_wg, void* out, hipStream_t st);
// workgroups [wg_first, wg_first + n_wg) of the plan: matrix units (row_tiles byte = kMatrixUnitRows)
hipError_t launch_attention_units_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan,
                                       int wg_first, int n_wg, int n_cand, PartialBuf part, hipStream_t st);
hipError_t launch_merge(const Shape& s, const PlanDev& plan, PartialBuf part, const void* q, const void* cand_k,
                        const void* cand_v, const uint8_t* mask, int n_cand, void* out, hipStream_t st);


}  // namespace apar
