// Partial decode attention over bf16 KV tiles on the gfx950 matrix cores.
//
// One wavefront per work unit = (run of blocks shared by one set of threads,
// kv head).  The unit's query rows - every sharing thread x candidate x q head
// of the kv group - sit on the N side of 16x16 matrix-core tiles, the 16 token
// slots of a block on the M side:
//
//   S^T[token][row] = K[token][:] . Q[row][:]          4 x mfma_f32_16x16x32_bf16
//   O^T[dim][row]  += V^T[dim][token] . P^T[token][row] 8 x mfma_f32_16x16x16_bf16
//
// K and V^T are the A operands and arrive straight from HBM in operand order
// (see the layout note in apar_internal.hpp): eight 16-byte loads per lane per
// tile, each a contiguous 1 KiB per wavefront.  The accumulator layout of S^T
// (lane = 16*g + c holds tokens 4g..4g+3 of row c) is already the B-operand
// layout of P^T, so the probabilities never move between lanes.  A block read
// once serves every row of the unit: that is where sibling threads reuse their
// shared prefix.
//
// Per row the kernel keeps a running maximum m (base-2 logits), a running sum l
// and the unnormalised output; it writes them as one partial result per
// (unit, row), which the merge kernel folds along each thread's root path.
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

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

__device__ __forceinline__ void load_tile(Frag (&k)[4], Frag (&v)[4], const char* tile, int lane) {
    const u32x4* p = reinterpret_cast<const u32x4*>(tile) + lane;
#pragma unroll
    for (int r = 0; r < 4; ++r) k[r].u = __builtin_nontemporal_load(p + r * 64);
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r].u = __builtin_nontemporal_load(p + 256 + r * 64);
}

template <int NT>
__global__ __launch_bounds__(256) void attention_partial_bf16(const char* __restrict__ pool,
                                                              const uint16_t* __restrict__ q, PlanDev plan,
                                                              int unit_begin, int unit_count, int n_cand, int n_q,
                                                              int n_kv, int group, float scale_log2e,
                                                              PartialBuf part) {
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (w >= unit_count * n_kv) return;
    const int kvh = w % n_kv;
    const UnitDesc u = plan.units[unit_begin + w / n_kv];
    const int g4 = lane >> 4, c = lane & 15;
    const int rows = u.n_shr * n_cand * group;

    // query rows -> B operands of the K.Q^T products; rows past the end are zero
    Frag qf[NT][4];
    int64_t slot[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = nt * 16 + c;
        slot[nt] = -1;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[nt][kk].u = u32x4{0u, 0u, 0u, 0u};
        if (row < rows) {
            const int gi = row % group, cc = (row / group) % n_cand, s = row / (group * n_cand);
            const int listed = plan.sharers[u.shr_ofs + s];
            const int hq = kvh * group + gi;
            const u32x4* qp = reinterpret_cast<const u32x4*>(q + (((int64_t)listed * n_cand + cc) * n_q + hq) * 128 +
                                                             g4 * 32);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qf[nt][kk].u = qp[kk];
            slot[nt] = ((int64_t)(u.part_base + s) * n_cand + cc) * n_q + hq;
        }
    }

    f32x4 o[NT][8];
    float m[NT], l[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m[nt] = -INFINITY;
        l[nt] = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[nt][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    const int64_t tile_stride = 8192;
    const int32_t* blk = plan.blocks + u.blk_ofs;
    Frag kc[4], vc[4], kn[4], vn[4];
    load_tile(kc, vc, pool + ((int64_t)blk[0] * n_kv + kvh) * tile_stride, lane);

    for (int b = 0; b < u.n_blk; ++b) {
        const bool more = b + 1 < u.n_blk;
        if (more) load_tile(kn, vn, pool + ((int64_t)blk[b + 1] * n_kv + kvh) * tile_stride, lane);
        const int valid = more ? 16 : u.last_valid;
        if (valid < 16) {
            // slots past the fill count hold whatever the buffer held: clear their V so a
            // zero probability cannot meet a NaN
            const uint32_t m01 = (4 * g4 + 0 < valid ? 0x0000ffffu : 0u) | (4 * g4 + 1 < valid ? 0xffff0000u : 0u);
            const uint32_t m23 = (4 * g4 + 2 < valid ? 0x0000ffffu : 0u) | (4 * g4 + 3 < valid ? 0xffff0000u : 0u);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                vc[r].u.x &= m01;
                vc[r].u.y &= m23;
                vc[r].u.z &= m01;
                vc[r].u.w &= m23;
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kc[kk].b8, qf[nt][kk].b8, s, 0, 0, 0);
            float sv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) sv[i] = (4 * g4 + i < valid) ? s[i] * scale_log2e : -INFINITY;
            float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m[nt], mx);
            const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
            float p[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(sv[i] - m_new);
            l[nt] = l[nt] * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
            m[nt] = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int j = 0; j < 8; ++j) o[nt][j] *= alpha;
            }
            union {
                uint32_t w[2];
                s16x4 h;
            } pp;
            pp.w[0] = pack_bf16_rne(p[0], p[1]);
            pp.w[1] = pack_bf16_rne(p[2], p[3]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                o[nt][2 * r] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vc[r].h4[0], pp.h, o[nt][2 * r], 0, 0, 0);
                o[nt][2 * r + 1] =
                    __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vc[r].h4[1], pp.h, o[nt][2 * r + 1], 0, 0, 0);
            }
        }
        if (more) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                kc[r] = kn[r];
                vc[r] = vn[r];
            }
        }
    }

    // one partial result per row: unnormalised output, running max and sum
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float lt = l[nt];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (slot[nt] >= 0) {
            float* dst = part.o + slot[nt] * 128 + 4 * g4;
#pragma unroll
            for (int j = 0; j < 8; ++j) *reinterpret_cast<f32x4*>(dst + 16 * j) = o[nt][j];
            if (g4 == 0) {
                part.ml[slot[nt] * 2] = m[nt];
                part.ml[slot[nt] * 2 + 1] = lt;
            }
        }
    }
}

}  // namespace

int attention_max_rows_per_unit(const Shape&) { return 64; }

hipError_t launch_attention_partial_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan,
                                         int n_cand, PartialBuf part, hipStream_t st) {
    // unit classes by the number of 16-row tiles they carry: [0] up to 64 rows, [1] up to 32, [2] up to 16
    int begin = 0;
    for (int cls = 0; cls < 3; ++cls) {
        const int count = plan.class_count[cls];
        if (count > 0) {
            const int64_t waves = (int64_t)count * s.n_kv;
            const dim3 grid((unsigned)((waves + 3) / 4));
#define APAR_ATTN(NTV)                                                                                           \
    hipLaunchKernelGGL((attention_partial_bf16<NTV>), grid, dim3(256), 0, st, (const char*)pool,                 \
                       (const uint16_t*)q, plan, begin, count, n_cand, s.n_q, s.n_kv, s.group, s.scale_log2e, part)
            if (cls == 0) APAR_ATTN(4);
            else if (cls == 1) APAR_ATTN(2);
            else APAR_ATTN(1);
#undef APAR_ATTN
        }
        begin += count;
    }
    return hipGetLastError();
}

}  // namespace apar
