// Internal declarations shared by the host side and the kernels of libapar.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apar.h"

namespace apar {

constexpr int kBlockTokens = 16;

// ---------------------------------------------------------------------------
// Pool layout in HBM.
//
// The pool is [block][kv_head] tiles; a tile holds the K rows and then the V
// rows of the block's 16 token slots for that head.
//
// f32 pools: both halves are row-major [16][d].
//
// bf16 pools (d = 128; tile = 4 KiB of K + 4 KiB of V): both halves are stored
// in the order the 16x16 matrix-core instructions consume them, so a wavefront
// fills its operand registers with four fully coalesced 1 KiB loads per half
// and no shuffle or LDS pass.  With lane = 16*g + c (g = 0..3, c = 0..15) and
// load index r = 0..3, the 16 bytes at  r*1024 + lane*16  hold
//   K half: K[token c][dims 32*g + 8*r .. +8]               (A operand of K.Q^T)
//   V half: V[tokens 4*g .. 4*g+3][dim 32*r + c] followed by
//           V[tokens 4*g .. 4*g+3][dim 32*r + 16 + c]       (A operand of V^T.P^T)
// ---------------------------------------------------------------------------
__host__ __device__ inline int bf16_k_offset(int token, int dim) {  // byte offset inside the K half
    return ((dim & 31) >> 3) * 1024 + (((dim >> 5) * 16 + token) * 16) + (dim & 7) * 2;
}
__host__ __device__ inline int bf16_v_offset(int token, int dim) {  // byte offset inside the V half
    return (dim >> 5) * 1024 + (((token >> 2) * 16 + (dim & 15)) * 16) + ((dim >> 4) & 1) * 8 + (token & 3) * 2;
}

// One work unit family: a run of blocks read for one set of sharing threads.
// The kernels launch one unit per (UnitDesc, kv head).
struct UnitDesc {
    int32_t blk_ofs;     // first entry in the flat block-id array
    int32_t n_blk;       // blocks in the run (>= 1)
    int32_t last_valid;  // filled slots in the run's last block (1..16); all others are full
    int32_t shr_ofs;     // first entry in the flat sharer array (indices into the listed threads)
    int32_t n_shr;       // threads sharing the run (rows = n_shr * n_cand * group size)
    int32_t part_base;   // first partial-result row of this unit
};

// A unit of at most 16 query rows and at most 8 blocks, self-contained in 64 bytes so
// that one scalar load tells a wavefront everything it needs to start streaming.
constexpr int kNarrowBlocks = 8;
struct NarrowDesc {
    int32_t n_blk;       // 1..8
    int32_t last_valid;  // filled slots of the last block
    int32_t n_shr;       // threads sharing the run
    int32_t part_base;   // first partial-result row
    int32_t shr;         // n_shr == 1: the listed-thread index itself; else first entry in the sharer array
    int32_t pad[3];
    int32_t blk[kNarrowBlocks];
};

struct PlanDev {              // device pointers of one staged plan
    const UnitDesc* units;    // all units; bf16 pools: the wide ones first, then the narrow ones
    const NarrowDesc* narrow; // bf16 pools: the narrow units again, in the same order, in their own format
    const int32_t* blocks;    // flat block ids
    const int32_t* sharers;   // flat listed-thread indices
    const int32_t* path_ofs;  // [n_threads + 1]
    const int32_t* path_ids;  // partial-result rows on each listed thread's root path
    int32_t n_units;          // UnitDesc count
    int32_t n_wide;           // units carrying more than 16 query rows (longest runs first)
    int32_t n_narrow;         // units carrying at most 16 (longest first)
    int32_t n_threads;
};

struct Shape {
    int32_t n_q, n_kv, d, group;  // group = n_q / n_kv
    int32_t dtype;
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

// ---- launchers (defined next to their kernels) ------------------------------
hipError_t launch_append_rows(const Shape& s, void* pool, const void* k, const void* v, const int32_t* dst_codes,
                              int n_rows, hipStream_t st);
hipError_t launch_block_copies(const Shape& s, void* pool, const int32_t* src_dst_pairs, int n_pairs,
                               hipStream_t st);
hipError_t launch_read_rows(const Shape& s, const void* pool, const int32_t* src_codes, int n_rows, void* k_out,
                            void* v_out, hipStream_t st);
hipError_t launch_attention_partial(const Shape& s, const void* pool, const void* q, const PlanDev& plan, int n_cand,
                                    int max_rows, PartialBuf part, hipStream_t st);
hipError_t launch_merge(const Shape& s, const PlanDev& plan, PartialBuf part, const void* q, const void* cand_k,
                        const void* cand_v, const uint8_t* mask, int n_cand, void* out, hipStream_t st);

// Largest number of query rows (threads * candidates * group) one unit may carry.
int attention_max_rows_per_unit(const Shape& s);

}  // namespace apar
