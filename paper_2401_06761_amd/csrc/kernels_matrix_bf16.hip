// Attention shaped for the matrix cores (bf16 pools): 32x32 products, 128 query rows per workgroup.
//
// Two kernels share one walk:
//   * prefill_bf16: a workgroup takes up to 128 query rows of ONE thread - consecutive query tokens x the
//     q heads of one kv group - and walks that thread's root path under the causal paragraph-tree mask;
//   * attention_units_bf16: a workgroup takes up to 128 query rows of threads that all hold one shared
//     segment (a decode step's stand-alone unit with many rows) and walks a chunk of that segment's
//     blocks; every row sees every filled slot, and the rows' softmax states go out as partial results.
//
// The walk goes in super-blocks of 32 token slots (two KV blocks).  Every wavefront owns 32 rows as the
// N side of 32x32 products:
//
//   S^T[token][row] = K[token][:] . Q[row][:]            8 x mfma_f32_32x32x16_bf16 per super-block
//   O^T[dim][row]  += V^T[dim][token] . P^T[token][row]   8 x mfma_f32_32x32x16_bf16 per super-block
//
// so a lane holds 16 logits per super-block and the per-tile bookkeeping of the online softmax (row
// maximum, the branch that moves the reference, sums) is spread over four times as many elements as in
// the row-tile kernel, and both products run at the full matrix rate.  The accumulator layout of S^T
// (lane = 32 h + n holds tokens 8 j + 4 h + i of row n) is the B-operand layout of P^T once the token
// index of the second product is permuted the same way, so probabilities never move between lanes.
//
// The four wavefronts share the path through LDS in groups of two super-blocks (four KV blocks, double
// buffered, one barrier per group): each wavefront fetches one block of the group while the previous
// group is consumed.  K is staged as it lies in HBM - operand order for a sealed block, row-major for a
// still open one (only the last block of a walk can be) - and read back with the matching address
// pattern; V is rearranged on its way into LDS so that an operand (8 token slots of one dim) is one
// 16-byte read.  Masks only matter at the end of a row's range: a super-block wholly below a
// wavefront's first limit is applied without masks, one wholly above its last limit is skipped.
#include <hip/hip_runtime.h>

#include "apar_internal.hpp"

namespace apar {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

union Op {  // 16 bytes: a load, or an 8-wide bf16 operand
    u32x4 u;
    bf16x8 b8;
};

constexpr float kSlack = 8.0f;      // a probability may exceed 1 by at most 2^kSlack before the reference moves
constexpr int kTileBytes = 8192;    // one (block, kv head): 4 KiB of K, 4 KiB of V
constexpr int kHalf = 4096;
constexpr int kBufBytes = 4 * kTileBytes;  // one staged group: four blocks, each K half then V half

__device__ __forceinline__ uint32_t pack_pair(float lo, float hi) {  // round to nearest even
    const f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Where the V operand of (matrix row block r = dims 32r.., dim 16 * hf + c, lane half h) lives inside a staged V
// half: 16 bytes = token slots 4h..4h+3 then 8+4h..8+4h+3 of that dim.  The sixteen lanes of one c run read
// 256 consecutive bytes.
__device__ __forceinline__ int v_operand_offset(int r, int hf, int c, int h) { return ((((r * 2 + hf) * 2 + h) * 16) + c) * 16; }

// What a wavefront brings to the walk.  `len` token slots are filled along the walk's block list
// (entry i of the list is table[i * table_stride]); the lane's row sees slots 0 .. pos.
struct Walk {
    const char* head_base;   // the pool at this kv head
    int64_t block_stride;
    const int32_t* table;
    int table_stride;
    int n_blk;               // blocks that hold a slot some row of the workgroup sees
    int len;
    bool wave_ok;            // the wavefront has rows at all
    int w_first, w_last;     // smallest and largest pos over the wavefront's rows (wavefront-uniform)
    bool row_ok;
    int pos;
    const uint16_t* q_row;   // the lane's query row (any valid row if !row_ok)
    float scale_log2e;
};

// Runs the walk; leaves the lane's share of O^T (dims 32 jj + 8 (i / 4) + 4 h + i % 4 of row n in o[jj][i]),
// the row's reference m and this lane's half of the row's sum l.
__device__ __forceinline__ void walk_blocks(const Walk& wk, char* lds, f32x16 (&o)[4], float& m, float& l) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 31, h = lane >> 5;   // column (query row) and half of the 32x32 products
    const int g4 = lane >> 4, c = lane & 15;  // the (token group, column) view of a sealed block's 16-byte pieces
    const char* head_base = wk.head_base;
    const int64_t block_stride = wk.block_stride;
    const bool wave_ok = wk.wave_ok, row_ok = wk.row_ok;
    const int w_first = wk.w_first, w_last = wk.w_last, pos = wk.pos;
    const float scale_log2e = wk.scale_log2e;

    // Q as the B operand: lane (n, h) holds dims 8 (2 s + h) .. + 8 of its row for product step s
    Op qv[8];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(wk.q_row);
#pragma unroll
        for (int s = 0; s < 8; ++s) qv[s].u = row_ok ? qp[2 * s + h] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[jj][i] = 0.0f;
    m = -INFINITY, l = 0.0f;

    // groups of four blocks (64 token slots)
    const int n_blk = wk.n_blk;
    const int n_grp = (n_blk + 3) / 4;
    // this wavefront stages block `wave` of every group
    u32x4 sk[4], sv[4];
    auto fetch = [&](int g) {
        // a group's last blocks may lie past the walk's last block: they are masked, re-read the last one
        const int blk = min(4 * g + wave, n_blk - 1);
        const int fill = min(16, wk.len - blk * 16);
        const char* tile = head_base + wk.table[blk * wk.table_stride] * block_stride;
        if (fill == 16) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sk[r] = *reinterpret_cast<const u32x4*>(tile + r * 1024 + lane * 16);
                sv[r] = *reinterpret_cast<const u32x4*>(tile + kHalf + r * 1024 + lane * 16);
            }
        } else {
            // the walk's last block is still open: row-major.  Piece r of this lane belongs to token row
            // 4r + g4; rows past the fill count re-read row 0 (finite values under probability 0)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int trow = 4 * r + g4 < fill ? 4 * r + g4 : 0;
                sk[r] = *reinterpret_cast<const u32x4*>(tile + trow * 256 + c * 16);
                sv[r] = *reinterpret_cast<const u32x4*>(tile + kHalf + trow * 256 + c * 16);
            }
        }
    };
    auto stage = [&](int g, char* buf) {
        const int blk = min(4 * g + wave, n_blk - 1);
        const bool sealed = wk.len - blk * 16 >= 16;
        char* dst = buf + wave * kTileBytes;
        // K: as it lies in HBM (either layout keeps piece r of lane l at r * 1024 + l * 16)
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<u32x4*>(dst + r * 1024 + lane * 16) = sk[r];
        dst += kHalf;
        if (sealed) {
            // V, sealed: piece r of lane (g4, c) = slots 4g4..4g4+3 of dim 32r + c, then of dim 32r + 16 + c
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const u32x2 lo = {sv[r].x, sv[r].y}, hi = {sv[r].z, sv[r].w};
                *reinterpret_cast<u32x2*>(dst + v_operand_offset(r, 0, c, g4 & 1) + 8 * (g4 >> 1)) = lo;
                *reinterpret_cast<u32x2*>(dst + v_operand_offset(r, 1, c, g4 & 1) + 8 * (g4 >> 1)) = hi;
            }
        } else {
            // V, open: piece r of this lane = slot 4r + g4, dims 8c .. 8c + 7
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = 4 * r + g4;
                const uint32_t w[4] = {sv[r].x, sv[r].y, sv[r].z, sv[r].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int dim = 8 * c + e;
                    const uint16_t val = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                    *reinterpret_cast<uint16_t*>(dst + v_operand_offset(dim >> 5, (dim >> 4) & 1, dim & 15, (slot >> 2) & 1) +
                                                 8 * (slot >> 3) + 2 * (slot & 3)) = val;
                }
            }
        }
    };

    fetch(0);
    stage(0, lds);
    if (n_grp > 1) fetch(1);
    __syncthreads();
    for (int g = 0; g < n_grp; ++g) {
        const char* buf = lds + (g & 1) * kBufBytes;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int t0 = 64 * g + 32 * sub;  // first token slot of the super-block
            if (!(wave_ok && t0 <= w_last)) continue;
            // ---- S^T = K . Q^T -------------------------------------------------------------------
            f32x16 s;
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = 0.0f;
            {
                // lane (n as token slot m, h): block m / 16 of the super-block, slot m % 16 of it
                const int j = 2 * sub + (n >> 4);
                const int blk = min(4 * g + j, n_blk - 1);
                const bool sealed = wk.len - blk * 16 >= 16;
                const char* kb = buf + j * kTileBytes;
                const int slot = n & 15;
                // all eight operands are requested before the first product waits for one
                Op a[8];
#pragma unroll
                for (int step = 0; step < 8; ++step) {
                    const int piece = 2 * step + h;  // dims 8 piece .. + 8
                    const int ofs = sealed ? (piece & 3) * 1024 + ((piece >> 2) * 16 + slot) * 16 : slot * 256 + piece * 16;
                    a[step].u = *reinterpret_cast<const u32x4*>(kb + ofs);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int step = 0; step < 8; ++step) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[step].b8, qv[step].b8, s, 0, 0, 0);
            }
            // the V operands travel from LDS while the softmax runs
            Op va[2][4];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)  // lane (n as dim 32 jj + n, h)
                    va[T][jj].u = *reinterpret_cast<const u32x4*>(buf + (2 * sub + T) * kTileBytes + kHalf +
                                                                  v_operand_offset(jj, n >> 4, n & 15, h));
            __builtin_amdgcn_sched_barrier(0);
            // ---- mask near the rows' limits: slot t0 + 8 (i / 4) + 4 h + i % 4 is visible up to the row's pos
            if (t0 + 31 > w_first) {
                const int room = row_ok ? pos - t0 - 4 * h : -1;  // visible iff 8 (i / 4) + i % 4 <= room
#pragma unroll
                for (int i = 0; i < 16; ++i) s[i] = (8 * (i >> 2) + (i & 3) <= room) ? s[i] : -INFINITY;
            }
            // ---- online softmax ------------------------------------------------------------------
            float top = s[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) top = fmaxf(top, s[i]);
            top = row_ok ? top * scale_log2e : -INFINITY;
            if (__builtin_amdgcn_ballot_w64(top > m + kSlack) != 0) {
                // some row ran away from its reference (always so on a row's first super-block): move every
                // row's reference to its running maximum (the two lanes of a row agree on it) and rescale
                const float mx = fmaxf(top, __shfl_xor(top, 32, 64));
                const float m_new = fmaxf(m, mx);
                const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
                l *= alpha;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[jj][i] *= alpha;
                m = m_new;
            }
            const float bias = (row_ok && m != -INFINITY) ? -m : -INFINITY;
            float p[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2e, bias));
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += p[i];
            l += sum;
            // ---- O^T += V^T . P^T: block T of the super-block uses elements 8T .. 8T + 7 ---------------
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                Op b;
                b.u.x = pack_pair(p[8 * T + 0], p[8 * T + 1]);
                b.u.y = pack_pair(p[8 * T + 2], p[8 * T + 3]);
                b.u.z = pack_pair(p[8 * T + 4], p[8 * T + 5]);
                b.u.w = pack_pair(p[8 * T + 6], p[8 * T + 7]);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) o[jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[T][jj].b8, b.b8, o[jj], 0, 0, 0);
            }
        }
        // hand over: the next group (in registers) goes into the other buffer, which everyone finished
        // reading before the barrier that ended the previous iteration
        if (g + 1 < n_grp) {
            stage(g + 1, lds + ((g + 1) & 1) * kBufBytes);
            if (g + 2 < n_grp) fetch(g + 2);
        }
        __syncthreads();
    }

}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void prefill_bf16(
    const char* __restrict__ pool, const uint16_t* __restrict__ q, const PrefillWg* __restrict__ wgs,
    const int32_t* __restrict__ tables, int n_q, int n_kv, int group, float scale_log2e, uint16_t* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) char lds[2 * kBufBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 31, h = lane >> 5;
    const int kvh = blockIdx.x % n_kv;
    const PrefillWg wg = wgs[blockIdx.x / n_kv];

    // this lane's query row: token tq of the workgroup's chunk, q head hg of the kv group
    const int row = wave * 32 + n;
    const int tq = row / group, hg = row - tq * group;
    const int w_tok0 = (wave * 32) / group;
    Walk wk;
    wk.head_base = pool + (int64_t)kvh * kTileBytes;
    wk.block_stride = (int64_t)n_kv * kTileBytes;
    wk.table = tables + wg.table_ofs;
    wk.table_stride = 1;
    wk.n_blk = (wg.p0 + wg.n_tok - 1) / 16 + 1;  // blocks that hold an attended token
    wk.len = wg.len;
    wk.row_ok = tq < wg.n_tok;
    wk.pos = wg.p0 + (wk.row_ok ? tq : 0);  // position of the row's token in the thread
    // first and last query position of the wavefront
    wk.wave_ok = w_tok0 < wg.n_tok;
    wk.w_first = wg.p0 + w_tok0;
    wk.w_last = wg.p0 + min(wg.n_tok - 1, (wave * 32 + 31) / group);
    const int64_t qrow = ((int64_t)(wg.q_row0 + (wk.row_ok ? tq : 0)) * n_q) + kvh * group + hg;
    wk.q_row = q + qrow * 128;
    wk.scale_log2e = scale_log2e;
    f32x16 o[4];
    float m, l;
    walk_blocks(wk, lds, o, m, l);

    // normalise and write
    const float lt = l + __shfl_xor(l, 32, 64);
    if (!wk.row_ok) return;
    const float inv = 1.0f / lt;
    uint16_t* dst = out + qrow * 128 + 4 * h;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u32x2 pk;
            pk.x = pack_pair(o[jj][4 * j + 0] * inv, o[jj][4 * j + 1] * inv);
            pk.y = pack_pair(o[jj][4 * j + 2] * inv, o[jj][4 * j + 3] * inv);
            __builtin_nontemporal_store(pk, reinterpret_cast<u32x2*>(dst + 32 * jj + 8 * j));
        }
}

// Stand-alone units of a decode plan with many rows.  The workgroup descriptor's shared tile list is the
// chunk of the segment (full blocks first, the open one last); its first wavefront entry names the
// threads: depth-first ranks grp_lo / n_slices .. + n_grp / n_slices, rows_per_thread rows each, laid
// flat over the 128 rows; part_base is the first thread's partial-result row for this chunk.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attention_units_bf16(
    const char* __restrict__ pool, const uint16_t* __restrict__ q, PlanDev plan, int wg_first, int n_cand, int n_q,
    int n_kv, int group, float scale_log2e, PartialBuf part) {
    __shared__ __attribute__((aligned(16))) char lds[2 * kBufBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 31, h = lane >> 5;
    const int kvh = blockIdx.x % n_kv;
    const WgDesc* wg = plan.wgs + wg_first + blockIdx.x / n_kv;
    const TileRef* tiles = plan.tiles + wg->coop_ofs;
    const int n_blk = wg->n_coop;
    const int rpt = plan.rows_per_thread;
    const int rank0 = wg->w[0].grp_lo / plan.n_slices, n_thr = wg->w[0].n_grp / plan.n_slices;
    const int last_fill = (tiles[n_blk - 1].meta >> 20) & 31;

    const int row = wave * 32 + n;
    const int tr = row / rpt, within = row - tr * rpt;
    Walk wk;
    wk.head_base = pool + (int64_t)kvh * kTileBytes;
    wk.block_stride = (int64_t)n_kv * kTileBytes;
    wk.table = &tiles[0].blk;
    wk.table_stride = sizeof(TileRef) / sizeof(int32_t);
    wk.n_blk = n_blk;
    wk.len = (n_blk - 1) * 16 + last_fill;
    wk.row_ok = tr < n_thr;
    wk.pos = wk.len - 1;  // every row sees every filled slot
    wk.wave_ok = wave * 32 < n_thr * rpt;
    wk.w_first = wk.w_last = wk.len - 1;
    const int tr_ok = wk.row_ok ? tr : 0, within_ok = wk.row_ok ? within : 0;
    const int listed = plan.dfs_threads ? plan.dfs_threads[rank0 + tr_ok] : rank0 + tr_ok;
    const int cc = within_ok / group, hq = kvh * group + (within_ok - cc * group);
    wk.q_row = q + (((int64_t)listed * n_cand + cc) * n_q + hq) * 128;
    wk.scale_log2e = scale_log2e;
    f32x16 o[4];
    float m, l;
    walk_blocks(wk, lds, o, m, l);

    // the row's state goes out as a partial result (streaming stores: read once, by the merge kernel)
    const float lt = l + __shfl_xor(l, 32, 64);
    if (!wk.row_ok) return;
    const int64_t slot = ((int64_t)(wg->w[0].part_base + tr) * n_cand + cc) * n_q + hq;
    float* dst = part.o + slot * 128 + 4 * h;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 v = {o[jj][4 * j + 0], o[jj][4 * j + 1], o[jj][4 * j + 2], o[jj][4 * j + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + 32 * jj + 8 * j));
        }
    if (h == 0) {
        __builtin_nontemporal_store(m, part.ml + slot * 2);
        __builtin_nontemporal_store(lt, part.ml + slot * 2 + 1);
    }
}

}  // namespace

hipError_t launch_prefill_bf16(const Shape& s, const void* pool, const void* q, const PrefillWg* wgs,
                               const int32_t* tables, int n_wg, void* out, hipStream_t st) {
    if (n_wg <= 0) return hipSuccess;
    const int64_t grid = (int64_t)n_wg * s.n_kv;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prefill_bf16, dim3((unsigned)grid), dim3(256), 0, st, (const char*)pool, (const uint16_t*)q, wgs,
                       tables, s.n_q, s.n_kv, s.group, s.scale_log2e, (uint16_t*)out);
    return hipGetLastError();
}

hipError_t launch_attention_units_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan,
                                       int wg_first, int n_wg, int n_cand, PartialBuf part, hipStream_t st) {
    if (n_wg <= 0) return hipSuccess;
    const int64_t grid = (int64_t)n_wg * s.n_kv;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attention_units_bf16, dim3((unsigned)grid), dim3(256), 0, st, (const char*)pool,
                       (const uint16_t*)q, plan, wg_first, n_cand, s.n_q, s.n_kv, s.group, s.scale_log2e, part);
    return hipGetLastError();
}

}  // namespace apar
