// Partial decode attention over bf16 KV tiles on the gfx950 matrix cores.
//
// A work unit is (run of blocks shared by one set of threads, kv head).  Its
// query rows - every sharing thread x candidate x q head of the kv group - sit
// on the N side of 16x16 matrix-core tiles, the 16 token slots of a block on
// the M side:
//
//   S^T[token][row] = K[token][:] . Q[row][:]          4 x mfma_f32_16x16x32_bf16
//   O^T[dim][row]  += V^T[dim][token] . P^T[token][row] 8 x mfma_f32_16x16x16_bf16
//
// K and V^T are the A operands and are stored in HBM in operand order (see the
// layout note in apar_internal.hpp): a wavefront fetches a tile half with four
// 16-byte loads per lane, each a contiguous 1 KiB.  The accumulator layout of
// S^T (lane = 16*g + c holds tokens 4g..4g+3 of row c) is already the
// B-operand layout of P^T, so probabilities never move between lanes.
//
// One launch, two kinds of workgroup (256 threads = 4 wavefronts):
//   * wide   - a unit with 17..64 rows, e.g. a prefix shared by many sibling
//              threads.  The four wavefronts fetch a quarter of each tile,
//              stage it in LDS (double buffered, one barrier per tile) and all
//              read it back from there; each applies it to its own 16 rows.
//              The shared block leaves HBM once and serves every sibling.
//   * narrow - four independent units of at most 16 rows and 8 blocks (private
//              tails, small groups), one per wavefront, tiles straight from
//              HBM into operand registers.
// Wide workgroups come first in the grid, so the launch tails off on the many
// short narrow units.
//
// Softmax runs in base 2 with a lazily updated reference: a row's reference
// logit m only moves when some logit exceeds it by more than kSlack, which
// keeps the cross-lane maximum and the rescale of the accumulators off the
// common path.  Each (unit, row) ends as one partial result (reference, sum,
// unnormalised output) that the merge kernel folds along the thread's root path.
#include <hip/hip_runtime.h>

#include "apar_internal.hpp"

namespace apar {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

union Frag {  // 16 bytes seen as a load, as an 8-wide bf16 operand, or as two 4-wide ones
    u32x4 u;
    bf16x8 b8;
    s16x4 h4[2];
};

constexpr float kSlack = 8.0f;  // a probability may exceed 1 by at most 2^kSlack before the reference moves
constexpr int kTileBytes = 8192;

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

// Rows of one wavefront: query operands, running softmax state, partial-result slot.
struct RowState {
    Frag q[4];
    f32x4 o[8];
    float m, l;
    int64_t slot;  // -1: this lane's row does not exist
};

__device__ __forceinline__ void init_rows(RowState& st, const uint16_t* __restrict__ q, const int32_t* sharers,
                                          int shr, int n_shr, int part_base, int row0, int n_cand, int n_q, int group,
                                          int kvh, int lane) {
    const int g4 = lane >> 4, c = lane & 15;
    const int row = row0 + c;
    const int rows = n_shr * n_cand * group;
    st.slot = -1;
    st.m = -INFINITY;
    st.l = 0.0f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) st.q[kk].u = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) st.o[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (row < rows) {
        const int gi = row % group, cc = (row / group) % n_cand, s = row / (group * n_cand);
        const int listed = sharers ? sharers[shr + s] : shr;
        const int hq = kvh * group + gi;
        const u32x4* qp =
            reinterpret_cast<const u32x4*>(q + (((int64_t)listed * n_cand + cc) * n_q + hq) * 128 + g4 * 32);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) st.q[kk].u = qp[kk];
        st.slot = ((int64_t)(part_base + s) * n_cand + cc) * n_q + hq;
    }
}

// S^T = K.Q^T for one tile, scaled to base-2 logits; slots >= valid become -inf.
__device__ __forceinline__ void scores(const Frag (&k)[4], const RowState& st, float scale_log2e, int valid, int g4,
                                       float (&sv)[4]) {
    f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[kk].b8, st.q[kk].b8, s, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = s[i] * scale_log2e;
    if (valid < 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * g4 + i >= valid) sv[i] = -INFINITY;
    }
}

// Online softmax step and O^T += V^T.P^T for one tile.
__device__ __forceinline__ void accumulate(Frag (&v)[4], RowState& st, const float (&sv)[4], int valid, int g4) {
    const float top = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    if (__builtin_amdgcn_ballot_w64(top > st.m + kSlack) != 0) {
        // some row's logits ran away from its reference: move every row's reference to its
        // running maximum (the four lanes of a row agree on it) and rescale what was summed
        float mx = fmaxf(top, __shfl_xor(top, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(st.m, mx);
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);  // first tile: exp2(-inf) = 0
        st.l *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[j] *= alpha;
        st.m = m_new;
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(sv[i] - st.m);
    st.l += (p[0] + p[1]) + (p[2] + p[3]);
    if (valid < 16) {
        // slots past the fill count hold whatever the buffer held: clear their V so that a
        // zero probability cannot meet a NaN
        const uint32_t m01 = (4 * g4 + 0 < valid ? 0x0000ffffu : 0u) | (4 * g4 + 1 < valid ? 0xffff0000u : 0u);
        const uint32_t m23 = (4 * g4 + 2 < valid ? 0x0000ffffu : 0u) | (4 * g4 + 3 < valid ? 0xffff0000u : 0u);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            v[r].u.x &= m01;
            v[r].u.y &= m23;
            v[r].u.z &= m01;
            v[r].u.w &= m23;
        }
    }
    union {
        uint32_t w[2];
        s16x4 h;
    } pp;
    pp.w[0] = pack_bf16_rne(p[0], p[1]);
    pp.w[1] = pack_bf16_rne(p[2], p[3]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        st.o[2 * r] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v[r].h4[0], pp.h, st.o[2 * r], 0, 0, 0);
        st.o[2 * r + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v[r].h4[1], pp.h, st.o[2 * r + 1], 0, 0, 0);
    }
}

__device__ __forceinline__ void store_partial(const RowState& st, PartialBuf part, int lane) {
    const int g4 = lane >> 4;
    float lt = st.l;
    lt += __shfl_xor(lt, 16, 64);
    lt += __shfl_xor(lt, 32, 64);
    if (st.slot >= 0) {
        float* dst = part.o + st.slot * 128 + 4 * g4;
#pragma unroll
        // streaming stores: the partial results are read once, by the merge kernel
        for (int j = 0; j < 8; ++j) __builtin_nontemporal_store(st.o[j], reinterpret_cast<f32x4*>(dst + 16 * j));
        if (g4 == 0) {
            __builtin_nontemporal_store(st.m, part.ml + st.slot * 2);
            __builtin_nontemporal_store(lt, part.ml + st.slot * 2 + 1);
        }
    }
}

__global__ __launch_bounds__(256) void attention_partial_bf16(const char* __restrict__ pool,
                                                              const uint16_t* __restrict__ q, PlanDev plan,
                                                              int n_wide_wg, int n_cand, int n_q, int n_kv, int group,
                                                              float scale_log2e, PartialBuf part) {
    __shared__ __attribute__((aligned(16))) char stage[2][kTileBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int g4 = lane >> 4;
    RowState st;

    if ((int)blockIdx.x < n_wide_wg) {
        // ---- wide unit: the workgroup shares each tile through LDS ------------------------
        const int kvh = blockIdx.x % n_kv;
        const UnitDesc u = plan.units[blockIdx.x / n_kv];
        const int rows = u.n_shr * n_cand * group;
        init_rows(st, q, plan.sharers, u.shr_ofs, u.n_shr, u.part_base, wave * 16, n_cand, n_q, group, kvh, lane);
        const bool active = wave * 16 < rows;  // wavefronts without rows still help to fetch
        const int32_t* blk = plan.blocks + u.blk_ofs;
        // this wavefront's quarter of a tile: K load index `wave` and V load index `wave`
        const int my_ofs = wave * 1024 + lane * 16;
        auto fetch = [&](int b, u32x4& kq, u32x4& vq) {
            const char* tile = pool + ((int64_t)blk[b] * n_kv + kvh) * kTileBytes;
            kq = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + my_ofs));
            vq = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 4096 + my_ofs));
        };
        u32x4 kq, vq;
        fetch(0, kq, vq);
        *reinterpret_cast<u32x4*>(&stage[0][my_ofs]) = kq;
        *reinterpret_cast<u32x4*>(&stage[0][4096 + my_ofs]) = vq;
        __syncthreads();
        for (int b = 0; b < u.n_blk; ++b) {
            const bool more = b + 1 < u.n_blk;
            if (more) fetch(b + 1, kq, vq);
            if (active) {
                const char* sb = stage[b & 1];
                const int valid = more ? 16 : u.last_valid;
                Frag k[4], v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) k[r].u = *reinterpret_cast<const u32x4*>(sb + r * 1024 + lane * 16);
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r].u = *reinterpret_cast<const u32x4*>(sb + 4096 + r * 1024 + lane * 16);
                float sv[4];
                scores(k, st, scale_log2e, valid, g4, sv);
                accumulate(v, st, sv, valid, g4);
            }
            if (more) {
                char* nb = stage[(b + 1) & 1];
                *reinterpret_cast<u32x4*>(nb + my_ofs) = kq;
                *reinterpret_cast<u32x4*>(nb + 4096 + my_ofs) = vq;
            }
            __syncthreads();  // tile b+1 is staged, and everyone is done reading tile b
        }
        if (active) store_partial(st, part, lane);
        return;
    }

    // ---- narrow units: one per wavefront, tiles go straight to operand registers ----------
    const int w = __builtin_amdgcn_readfirstlane((int)((blockIdx.x - n_wide_wg) * 4) + wave);
    if (w >= plan.n_narrow * n_kv) return;
    const int kvh = w % n_kv;
    const NarrowDesc d = plan.narrow[w / n_kv];
    const u32x4* t0 = reinterpret_cast<const u32x4*>(pool + ((int64_t)d.blk[0] * n_kv + kvh) * kTileBytes) + lane;
    Frag k[4], v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) k[r].u = __builtin_nontemporal_load(t0 + r * 64);
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r].u = __builtin_nontemporal_load(t0 + 256 + r * 64);
    init_rows(st, q, d.n_shr == 1 ? nullptr : plan.sharers, d.shr, d.n_shr, d.part_base, 0, n_cand, n_q, group, kvh,
              lane);
    const int32_t* blk = plan.narrow[w / n_kv].blk;
    for (int b = 0; b < d.n_blk; ++b) {
        const bool more = b + 1 < d.n_blk;
        const int valid = more ? 16 : d.last_valid;
        const u32x4* tn = nullptr;
        if (more) tn = reinterpret_cast<const u32x4*>(pool + ((int64_t)blk[b + 1] * n_kv + kvh) * kTileBytes) + lane;
        float sv[4];
        scores(k, st, scale_log2e, valid, g4, sv);
        if (more) {  // K registers are free again: start fetching the next tile's K
#pragma unroll
            for (int r = 0; r < 4; ++r) k[r].u = __builtin_nontemporal_load(tn + r * 64);
        }
        accumulate(v, st, sv, valid, g4);
        if (more) {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r].u = __builtin_nontemporal_load(tn + 256 + r * 64);
        }
    }
    store_partial(st, part, lane);
}

}  // namespace

int attention_max_rows_per_unit(const Shape&) { return 64; }

hipError_t launch_attention_partial_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan,
                                         int n_cand, PartialBuf part, hipStream_t st) {
    const int64_t wide_wg = (int64_t)plan.n_wide * s.n_kv;
    const int64_t narrow_wg = ((int64_t)plan.n_narrow * s.n_kv + 3) / 4;
    if (wide_wg + narrow_wg <= 0) return hipSuccess;
    if (wide_wg + narrow_wg > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attention_partial_bf16, dim3((unsigned)(wide_wg + narrow_wg)), dim3(256), 0, st,
                       (const char*)pool, (const uint16_t*)q, plan, (int)wide_wg, n_cand, s.n_q, s.n_kv, s.group,
                       s.scale_log2e, part);
    return hipGetLastError();
}

}  // namespace apar
