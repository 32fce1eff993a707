// Decode attention over bf16 KV tiles on the gfx950 matrix cores.
//
// Query rows - (thread, candidate, q head of one kv group) - sit on the N side
// of 16x16 matrix-core tiles, the 16 token slots of a block on the M side:
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
// A workgroup (4 wavefronts, 16 or 32 rows each) is given by the host plan
//   * a shared tile list: blocks whose holders sit in more than one wavefront
//     (prefixes shared by many sibling threads).  They go through LDS in groups
//     of four, one whole tile per wavefront, the next group in flight to
//     registers while the current one is consumed (two barriers per group), and
//     every wavefront applies each tile to those of its rows that hold the block;
//   * one private tile list per wavefront: blocks held only by rows of that
//     wavefront (private tails, small sibling groups), loaded straight from HBM
//     into operand registers with no barrier.  K registers are refilled right
//     after the K.Q^T products and V registers after the V^T.P^T products, so
//     the next tile is in flight while the current one is consumed.
// Every list holds its full tiles first: they run through loops with nothing
// but unconditional loads; the open tiles after them through general loops.
// Every tile names the range of row groups it applies to; other rows see -inf
// logits.  A causal tile (prefill: the query tokens are the row groups) shows
// each further row group one more of its token slots.  A row's softmax state stays in registers across all the blocks of
// its root path that the unit covers; attention is a set operation, so the
// order in which a unit visits them does not matter.  Rows whose whole path
// lies in the unit are normalised and written out here; the others leave a
// partial result (reference, sum, unnormalised output) for the merge kernel.
//
// A block that is still filling (fewer than 16 slots) is stored row-major, not in
// operand order; such tiles - at most one per segment - take a slower path: K
// pieces are gathered row by row and V goes through a padded LDS transpose.
//
// fp8 pools (template parameter F8): a full block holds fp8 codes in the same element order, half the
// bytes, and one power-of-two scale per half.  Its tiles are fetched with two 16-byte loads per lane and
// half and turned into the bf16 operands by the hardware conversion that multiplies by the scale (exact: a
// code times a power of two is a bf16 value) - private tiles on their way into the operand registers,
// shared tiles once, by the wavefront that stages them, so that LDS holds the bf16 tile.  Everything after
// that - products, softmax, accumulation - is the code of the bf16 pool.
// Blocks that are still filling are bf16 rows on either pool.
//
// Softmax runs in base 2 with a lazily updated reference: a row's reference
// logit m only moves when some logit exceeds it by more than kSlack, which
// keeps the cross-lane maximum and the rescale of the accumulators off the
// common path.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "apar_internal.hpp"

namespace apar {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

union Frag {  // 16 bytes seen as a load, as an 8-wide bf16 operand, or as two 4-wide ones
    u32x4 u;
    bf16x8 b8;
    s16x4 h4[2];
};

constexpr float kSlack = 8.0f;  // a probability may exceed 1 by at most 2^kSlack before the reference moves
constexpr int kTileBytes = 8192;

// The 16 rows of one wavefront: query operands and running softmax state.
struct RowState {
    Frag q[4];
    f32x4 o[8];
    float m, l;
};

// S^T = K.Q^T for one tile: raw dot products, tokens 4*g4 .. 4*g4+3 of this lane's row.
__device__ __forceinline__ f32x4 products(const Frag (&k)[4], const RowState& st) {
    f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[kk].b8, st.q[kk].b8, s, 0, 0, 0);
    return s;
}

// Token slots whose bit is clear in tok_mask (per lane, i.e. per query row) get a product of -inf and
// hence probability 0.  Only needed for tiles that are not full and for candidate tiles.
__device__ __forceinline__ void mask_tokens(f32x4& s, uint32_t tok_mask, int g4) {
    const uint32_t mine = tok_mask >> (4 * g4);
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = ((mine >> i) & 1u) ? s[i] : -INFINITY;
}

__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {  // round to nearest even, one instruction
    const f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Two 16-byte pieces of fp8 codes (one half of a sealed fp8 tile as this lane holds it) times the half's
// power-of-two scale -> the four bf16 operand pieces of the half.
__device__ __forceinline__ void fp8_operands(const u32x4 (&raw)[2], float scale, Frag (&f)[4]) {
#pragma unroll
    for (int rp = 0; rp < 2; ++rp)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            Frag& dst = f[2 * rp + (w >> 1)];
            dst.u[2 * (w & 1)] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[rp][w], scale, false));
            dst.u[2 * (w & 1) + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[rp][w], scale, true));
        }
}

// Online softmax step, first half: if some row's logits ran away from its reference (always so for a
// row's first tile, whose reference is still -inf), move every row's reference to its running maximum
// (the four lanes of a row agree on it) and rescale what was summed.  Rare, hence behind a branch.
__device__ __forceinline__ float top_logit(const f32x4& s, bool in_range, float scale_log2e) {
    return in_range ? fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])) * scale_log2e : -INFINITY;
}

__device__ __forceinline__ void raise_reference(RowState& st, float top) {
    float mx = fmaxf(top, __shfl_xor(top, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(st.m, mx);
    // a row that has seen nothing yet keeps m = -inf and sums of zero
    const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(st.m - m_new);
    st.l *= alpha;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.o[j] *= alpha;
    st.m = m_new;
}

__device__ __forceinline__ void move_reference(RowState& st, const f32x4& s, bool in_range, float scale_log2e) {
    const float top = top_logit(s, in_range, scale_log2e);
    if (__builtin_amdgcn_ballot_w64(top > st.m + kSlack) != 0) raise_reference(st, top);
}

// The same for all row tiles of a wavefront behind ONE branch (a branch on a vector compare costs
// the wavefront some eighty cycles): if any row of any tile ran away, every touched tile's rows move
// to their running maxima, which is always allowed.
template <int NT>
__device__ __forceinline__ void move_references(RowState (&st)[NT], const f32x4 (&s)[NT], const bool (&on)[NT],
                                                const bool (&in_range)[NT], float scale_log2e) {
    float top[NT];
    bool ran_away = false;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        top[nt] = on[nt] ? top_logit(s[nt], in_range[nt], scale_log2e) : -INFINITY;
        ran_away = ran_away || top[nt] > st[nt].m + kSlack;
    }
    if (__builtin_amdgcn_ballot_w64(ran_away) != 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (on[nt]) raise_reference(st[nt], top[nt]);
    }
}

// Second half, straight-line: probabilities and O^T += V^T.P^T for one tile that applies to this lane's
// row iff in_range.  The softmax scale and the reference are folded into one fused multiply-add per
// logit; rows outside the range, and slots masked to -inf, get probability exp2(-inf) = 0.  V rows of
// unfilled slots must be finite (the loaders hand over a copy of row 0 for them): 0 * V is added.
__device__ __forceinline__ void weigh_values(const Frag (&v)[4], RowState& st, const f32x4& s, bool in_range,
                                             float scale_log2e) {
    const float bias = (in_range && st.m != -INFINITY) ? -st.m : -INFINITY;
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2e, bias));
    st.l += (p[0] + p[1]) + (p[2] + p[3]);
    union {
        uint32_t w[2];
        s16x4 h;
    } pp;
    pp.w[0] = pack_bf16_pair(p[0], p[1]);
    pp.w[1] = pack_bf16_pair(p[2], p[3]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        st.o[2 * r] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v[r].h4[0], pp.h, st.o[2 * r], 0, 0, 0);
        st.o[2 * r + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v[r].h4[1], pp.h, st.o[2 * r + 1], 0, 0, 0);
    }
}

__device__ __forceinline__ void accumulate(const Frag (&v)[4], RowState& st, const f32x4& s, bool in_range,
                                           float scale_log2e) {
    move_reference(st, s, in_range, scale_log2e);
    weigh_values(v, st, s, in_range, scale_log2e);
}

// V^T operand pieces out of a ROW-MAJOR V half held in LDS (rows `stride` bytes apart):
// piece r holds V[tokens 4g..4g+3][dim 32r + c] and V[tokens 4g..4g+3][dim 32r + 16 + c].
__device__ __forceinline__ void v_operands_from_rows(const char* vrows, int stride, int g4, int c, Frag (&v)[4]) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const char* col = vrows + (32 * r + 16 * hh + c) * 2 + 4 * g4 * stride;
            const uint32_t a0 = *reinterpret_cast<const uint16_t*>(col);
            const uint32_t a1 = *reinterpret_cast<const uint16_t*>(col + stride);
            const uint32_t a2 = *reinterpret_cast<const uint16_t*>(col + 2 * stride);
            const uint32_t a3 = *reinterpret_cast<const uint16_t*>(col + 3 * stride);
            v[r].u[2 * hh] = a0 | (a1 << 16);
            v[r].u[2 * hh + 1] = a2 | (a3 << 16);
        }
    }
}

constexpr int kOpenRowStride = 264;                 // padded, so the four token groups hit different LDS banks
constexpr int kOpenScratch = 16 * kOpenRowStride;   // one wavefront's row-major V half

// NT = 16-row tiles per wavefront (1 or 2 are instantiated): a workgroup carries up to 64 * NT query rows.
// F8: full blocks hold fp8 codes and two scales (APAR_BF16_FP8KV pools).
template <int NT, bool F8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NT == 1 ? 3 : 2))) void attention_bf16(const char* __restrict__ pool, const uint16_t* __restrict__ q,
                                                      PlanDev plan, int wg_first, int n_cand, int n_q, int n_kv,
                                                      int group, float scale_log2e, PartialBuf part,
                                                      const uint16_t* __restrict__ cand_k,
                                                      const uint16_t* __restrict__ cand_v,
                                                      const uint8_t* __restrict__ cand_mask,
                                                      uint16_t* __restrict__ out) {
    // four staged tiles during the shared phase; then one V-transpose scratch per wavefront; last, three
    // wavefronts' row states when a unit is split
    __shared__ __attribute__((aligned(16))) char lds[4 * kTileBytes];
    static_assert(4 * kTileBytes >= 3 * 16 * 130 * 4 && 4 * kTileBytes >= 4 * kOpenScratch, "LDS areas overlap in time");
    char(*stage)[kTileBytes] = reinterpret_cast<char(*)[kTileBytes]>(lds);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int g4 = lane >> 4, c = lane & 15;
    const int kvh = blockIdx.x % n_kv;
    const WgDesc* wg = plan.wgs + wg_first + blockIdx.x / n_kv;
    const WaveItem wi = wg->w[wave];
    const int n_coop = wg->n_coop;
    const TileRef* coop = plan.tiles + wg->coop_ofs;
    const TileRef* mine = plan.tiles + wi.tile_ofs;
    const char* head_base = pool + (int64_t)kvh * kTileBytes;
    const int64_t block_stride = (int64_t)n_kv * kTileBytes;

    // Row geometry: column c of row tile nt is row `within` of the wavefront's row group nt * cap + c / rps.
    const int rps = plan.rows_per_slice, n_sl = plan.n_slices, rpt = plan.rows_per_thread;
    const int cap = 16 / rps;
    const int jc = c / rps, within = c - jc * rps;
    RowState st[NT];
    int my_j[NT];       // row group of this lane's row, relative to the wavefront's first; 0x7fff: no row
    // where the row of tile nt lives: depth-first rank of its thread, row within the thread's rows,
    // q/output row and partial-result slot (recomputed where needed rather than kept in registers)
    auto locate = [&](int nt, int& rank, int& rr, int64_t& qrow, int64_t& slot) {
        const int grp = wi.grp_lo + nt * cap + jc;
        rank = grp / n_sl;
        rr = (grp - rank * n_sl) * rps + within;
        const int listed = plan.dfs_threads ? plan.dfs_threads[rank] : rank;
        const int cc = rr / group, hq = kvh * group + (rr - cc * group);
        qrow = ((int64_t)listed * n_cand + cc) * n_q + hq;
        slot = ((int64_t)(wi.part_base + rank - wi.grp_lo / n_sl) * n_cand + cc) * n_q + hq;
    };
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int j = nt * cap + jc;
        const int grp = wi.grp_lo + j;
        const int rank = grp / n_sl, rr = (grp - rank * n_sl) * rps + within;
        const bool ok = jc < cap && j < wi.n_grp && rr < rpt;
        my_j[nt] = ok ? j : 0x7fff;
        st[nt].m = -INFINITY;
        st[nt].l = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) st[nt].q[kk].u = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) st[nt].o[jj] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (ok) {
            int rk, r2;
            int64_t qrow, slot;
            locate(nt, rk, r2, qrow, slot);
            const u32x4* qp = reinterpret_cast<const u32x4*>(q + qrow * 128 + g4 * 32);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) st[nt].q[kk].u = qp[kk];
        }
    }
    // token slots of a tile that the row `ahead` row groups past the tile's first one may see: the filled
    // ones; of a causal tile (bit 30) `first` slots (bits 25-29) for the first row group and one more for
    // every further one
    auto visible = [](int meta, int ahead) -> uint32_t {
        const int fill = (meta >> 20) & 31;
        const int limit = (meta >> 30) ? min(fill, max(0, ((meta >> 25) & 31) + ahead)) : fill;
        return (1u << limit) - 1u;
    };
    // does a tile touch row tile nt at all?  (wavefront-uniform)
    auto touches = [&](int nt, int lo, int hi) -> bool {
        return lo < min((nt + 1) * cap, wi.n_grp) && hi > nt * cap;
    };

    // Makes the query operands' loads known to have landed (an empty statement that names the registers:
    // the compiler must wait for them there).  Used once in front of the shared-tile loops.  Without it the
    // compiler's wait-count bookkeeping carries the query loads of the kernel's start into those loops as
    // if they were the youngest loads in flight, and every product waits for the tile prefetch issued just
    // before it, which defeats the prefetch.
    auto settle_queries = [&]() {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) asm("" : "+v"(st[nt].q[kk].u));
    };

    // ---- shared tiles: staged once in LDS for the whole workgroup ---------------------------
    // Tiles go through LDS in groups of four, one whole tile per wavefront: while a group is consumed
    // from LDS, each wavefront already has its tile of the next group in flight to its registers.
    // Full tiles (16 filled slots) come first in every list and go through a loop that contains no
    // lane-dependent branch around a load (which would make the compiler wait for each load where it is
    // issued); the open tiles after them go through a general loop.
    if (n_coop > 0) {
        const int shift = wi.grp_lo - wg->grp_base;  // shared ranges are relative to the group's base
        const int n_coop_full = wg->row_tiles >> 8;
        u32x4 rk[4], rv[4];
        // Shared tiles are fetched with plain loads, private ones (below) with non-temporal loads: a shared
        // tile may be read again by another workgroup (the units below an inlined segment all read it; so do
        // the stand-alone units of a segment with many rows) and is worth a place in L2, a private tile is
        // read exactly once.  Measured: plain loads here take 6-10 % off the HBM traffic of the speculative
        // loop and 2 % off the headline launch; plain loads for the private tiles cost 8 %.
        f32x2 rsc = {1.0f, 1.0f};  // fp8 pools: the scales of the tile in flight
        auto fetch_full = [&](int t) {
            const char* tile = head_base + coop[t].blk * block_stride + lane * 16;
            if constexpr (F8) {
#pragma unroll
                for (int rp = 0; rp < 2; ++rp) {
                    rk[rp] = *reinterpret_cast<const u32x4*>(tile + rp * 1024);
                    rv[rp] = *reinterpret_cast<const u32x4*>(tile + kFp8HalfBytes + rp * 1024);
                }
                rsc = *reinterpret_cast<const f32x2*>(tile - lane * 16 + kFp8ScaleOfs);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    rk[r] = *reinterpret_cast<const u32x4*>(tile + r * 1024);
                    rv[r] = *reinterpret_cast<const u32x4*>(tile + 4096 + r * 1024);
                }
            }
        };
        auto fetch_any = [&](int t) {
            if (t >= n_coop) return;
            const int fill = (coop[t].meta >> 20) & 31;
            if (!F8 && fill == 16) {  // (a list holds its full tiles first: none of them comes through here on an fp8 pool)
                fetch_full(t);
            } else {
                // an open block is row-major: piece r of this lane belongs to token row 4r + g4.  Rows past the
                // fill count are never read: their lanes re-read row 0 instead (same cache lines, no extra
                // traffic, no branch around a load); the masked logits give those slots probability 0.
                const char* tile = head_base + coop[t].blk * block_stride + c * 16;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 4 * r + g4 < fill ? 4 * r + g4 : 0;
                    rk[r] = *reinterpret_cast<const u32x4*>(tile + row * 256);
                    rv[r] = *reinterpret_cast<const u32x4*>(tile + 4096 + row * 256);
                }
            }
        };
        auto to_stage = [&](auto full_tile) {
            char* dst = stage[wave] + lane * 16;
            if constexpr (F8 && decltype(full_tile)::value) {
                // the codes are widened once, by the wavefront that fetched them: what is staged is the bf16 tile in
                // operand order, as on a bf16 pool, and the four consumers read it as such
                Frag ks[4], vs[4];
                const u32x4 kraw[2] = {rk[0], rk[1]}, vraw[2] = {rv[0], rv[1]};
                fp8_operands(kraw, rsc.x, ks);
                fp8_operands(vraw, rsc.y, vs);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    *reinterpret_cast<u32x4*>(dst + r * 1024) = ks[r].u;
                    *reinterpret_cast<u32x4*>(dst + 4096 + r * 1024) = vs[r].u;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    *reinterpret_cast<u32x4*>(dst + r * 1024) = rk[r];
                    *reinterpret_cast<u32x4*>(dst + 4096 + r * 1024) = rv[r];
                }
            }
        };
        // the operands of a staged full tile
        auto staged_operands = [&](const char* sb, Frag (&ks)[4], Frag (&vs)[4]) {
#pragma unroll
            for (int r = 0; r < 4; ++r) ks[r].u = *reinterpret_cast<const u32x4*>(sb + r * 1024 + lane * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) vs[r].u = *reinterpret_cast<const u32x4*>(sb + 4096 + r * 1024 + lane * 16);
        };
        auto consume = [&](int t, const char* sb, auto full_only) {
            constexpr bool kFull = decltype(full_only)::value;
            const int meta = coop[t].meta;
            const int lo = (meta & 1023) - shift, hi = ((meta >> 10) & 1023) - shift;
            const int valid = kFull ? 16 : (meta >> 20) & 31;
            // does the tile touch any row group of this wavefront?
            if (wi.n_grp == 0 || lo >= wi.n_grp || hi <= 0) return;
            Frag ks[4], vs[4];
            if (kFull || (!F8 && valid == 16)) {
                staged_operands(sb, ks, vs);
            } else {  // an open block: row-major in the stage buffer
#pragma unroll
                for (int r = 0; r < 4; ++r) ks[r].u = *reinterpret_cast<const u32x4*>(sb + c * 256 + g4 * 64 + r * 16);
                v_operands_from_rows(sb + 4096, 256, g4, c, vs);
            }
            // phase by phase over the row tiles, so that the products of one overlap the softmax of another
            f32x4 s[NT];
            bool on[NT], in_range[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                on[nt] = NT == 1 || touches(nt, lo, hi);
                in_range[nt] = my_j[nt] >= lo && my_j[nt] < hi;
                if (on[nt]) s[nt] = products(ks, st[nt]);
            }
            if ((!kFull && valid < 16) || (meta >> 30)) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (on[nt]) mask_tokens(s[nt], visible(meta, my_j[nt] - lo), g4);
            }
            move_references<NT>(st, s, on, in_range, scale_log2e);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (on[nt]) weigh_values(vs, st[nt], s[nt], in_range[nt], scale_log2e);
        };
        // A full tile that every row group of the workgroup sees (the segments at the top of a unit: the common
        // case) needs no range, no mask and no decision per row tile: straight-line code around one rare branch
        // (the move of the references), a dozen scalar branches and a scalar load fewer per tile than the
        // general code.  Measured: 4 % off a prefill call, under 1 % off the decode calls.
        // Such tiles are taken in a loop of their own - inside one loop, next to the general code, the two
        // paths would disagree on the accumulators' registers and every tile would end in 64 register moves.
        auto consume_seen_by_all = [&](const char* sb) {
            if (wi.n_grp == 0) return;
            Frag ks[4], vs[4];
            staged_operands(sb, ks, vs);
            f32x4 s[NT];
            float top[NT];
            bool ran_away = false;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s[nt] = products(ks, st[nt]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                top[nt] = top_logit(s[nt], my_j[nt] != 0x7fff, scale_log2e);
                ran_away = ran_away || top[nt] > st[nt].m + kSlack;
            }
            if (__builtin_amdgcn_ballot_w64(ran_away) != 0) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) raise_reference(st[nt], top[nt]);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) weigh_values(vs, st[nt], s[nt], my_j[nt] != 0x7fff, scale_log2e);
        };
        // Two such tiles at once: twice as many independent chains of matrix instructions and one decision
        // about the references instead of two (a wavefront spends most of its time between dependent
        // instructions, not in them).
        auto consume_two_seen_by_all = [&](const char* sa, const char* sb) {
            if (wi.n_grp == 0) return;
            Frag ka[4], kb[4], va[4], vb[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) ka[r].u = *reinterpret_cast<const u32x4*>(sa + r * 1024 + lane * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) kb[r].u = *reinterpret_cast<const u32x4*>(sb + r * 1024 + lane * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) va[r].u = *reinterpret_cast<const u32x4*>(sa + 4096 + r * 1024 + lane * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) vb[r].u = *reinterpret_cast<const u32x4*>(sb + 4096 + r * 1024 + lane * 16);
            f32x4 s0[NT], s1[NT];
            float top[NT];
            bool ran_away = false;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s0[nt] = products(ka, st[nt]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s1[nt] = products(kb, st[nt]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const bool mine = my_j[nt] != 0x7fff;
                top[nt] = fmaxf(top_logit(s0[nt], mine, scale_log2e), top_logit(s1[nt], mine, scale_log2e));
                ran_away = ran_away || top[nt] > st[nt].m + kSlack;
            }
            if (__builtin_amdgcn_ballot_w64(ran_away) != 0) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) raise_reference(st[nt], top[nt]);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                weigh_values(va, st[nt], s0[nt], my_j[nt] != 0x7fff, scale_log2e);
                weigh_values(vb, st[nt], s1[nt], my_j[nt] != 0x7fff, scale_log2e);
            }
        };
        if (n_coop_full > 0) {  // the full tiles; which wavefront fetches is a scalar decision
            if (wave < n_coop_full) fetch_full(wave);
            // how many tiles at the head of the list are seen by all (the same count in every wavefront)
            int n_all = 0;
            for (int k = 0; k < 4; ++k)
                if (wg->w[k].n_grp > 0) n_all = max(n_all, wg->w[k].grp_lo + wg->w[k].n_grp - wg->grp_base);
            int n_lead = 0;
            for (int base = 0; base < n_coop_full; base += 64) {
                bool seen_by_all = false;
                if (base + lane < n_coop_full) {
                    const int meta = coop[base + lane].meta;
                    seen_by_all = (meta & 1023) == 0 && ((meta >> 10) & 1023) >= n_all && !(meta >> 30);
                }
                const uint64_t others = ~__builtin_amdgcn_ballot_w64(seen_by_all);
                const int run = others == 0 ? 64 : __builtin_ctzll(others);
                n_lead += run;
                if (run < 64) break;
            }
            // whole groups of four, or the whole list
            const int n_fast = n_lead >= n_coop_full ? n_coop_full : (n_lead & ~3);
            settle_queries();
            int t0 = 0;
            for (; t0 < n_fast; t0 += 4) {
                if (t0 > 0) __syncthreads();  // everyone is done reading the previous group
                if (t0 + wave < n_coop_full) to_stage(std::true_type{});
                __syncthreads();
                if (t0 + 4 + wave < n_coop_full) fetch_full(t0 + 4 + wave);
                const int n_here = min(4, n_coop_full - t0);
                int u = 0;
                for (; u + 1 < n_here; u += 2) consume_two_seen_by_all(stage[u], stage[u + 1]);
                if (u < n_here) consume_seen_by_all(stage[u]);
            }
            for (; t0 < n_coop_full; t0 += 4) {
                if (t0 > 0) __syncthreads();
                if (t0 + wave < n_coop_full) to_stage(std::true_type{});
                __syncthreads();
                if (t0 + 4 + wave < n_coop_full) fetch_full(t0 + 4 + wave);
                const int n_here = min(4, n_coop_full - t0);
                for (int u = 0; u < n_here; ++u) consume(t0 + u, stage[u], std::true_type{});
            }
        }
        if (n_coop_full < n_coop) {  // the open tiles
            if (n_coop_full > 0) __syncthreads();
            fetch_any(n_coop_full + wave);
            settle_queries();
            for (int t0 = n_coop_full; t0 < n_coop; t0 += 4) {
                if (t0 > n_coop_full) __syncthreads();
                if (t0 + wave < n_coop) to_stage(std::false_type{});
                __syncthreads();
                fetch_any(t0 + 4 + wave);
                const int n_here = min(4, n_coop - t0);
                for (int u = 0; u < n_here; ++u) consume(t0 + u, stage[u], std::false_type{});
            }
        }
        __syncthreads();  // the stage buffers are reused below
    }
    if (wi.n_grp == 0) return;  // a wavefront without rows only helped to fetch

    // ---- private tiles: straight into operand registers -------------------------------------
    // K pieces of a sealed tile are 1 KiB apart with the lanes side by side; of an open tile, 16 bytes
    // apart inside the lane's own 64 bytes of its token's row.  The V half is fetched raw either way.
    // K registers are refilled right after the K.Q^T products and V registers after the V^T.P^T products.
    Frag k[4], v[4];
    // fp8 pools: the codes of a full tile's halves as fetched, and the halves' scales; they become k, v just
    // before use (k_ready, v_ready), so that the codes of the next tile can be in flight meanwhile
    u32x4 k8[2], v8[2];
    float k8s = 1.0f, v8s = 1.0f;
    auto issue_k_full = [&](const char* tile) {
        const char* p = tile + lane * 16;
        if constexpr (F8) {
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) k8[rp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + rp * 1024));
            k8s = *reinterpret_cast<const float*>(tile + kFp8ScaleOfs);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) k[r].u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + r * 1024));
        }
    };
    auto issue_v_full = [&](const char* tile) {
        if constexpr (F8) {
            const char* p = tile + kFp8HalfBytes + lane * 16;
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) v8[rp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + rp * 1024));
            v8s = *reinterpret_cast<const float*>(tile + kFp8ScaleOfs + 4);
        } else {
            const u32x4* p = reinterpret_cast<const u32x4*>(tile + 4096) + lane;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r].u = __builtin_nontemporal_load(p + r * 64);
        }
    };
    auto k_ready = [&](int valid) {  // (valid is wavefront-uniform)
        if constexpr (F8)
            if (valid == 16) fp8_operands(k8, k8s, k);
    };
    auto v_ready = [&](int valid) {
        if constexpr (F8)
            if (valid == 16) fp8_operands(v8, v8s, v);
    };
    // Only the filled rows of an open tile are read: a lane whose row lies past the fill count re-reads
    // row 0 (no branch around the loads, no extra traffic), and the masked logits give the slot probability 0.
    auto issue_k = [&](const char* tile, int valid) {
        if (valid == 16) {
            issue_k_full(tile);
        } else {
            const char* p = tile + (c < valid ? c : 0) * 256 + g4 * 64;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                k[r].u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + r * 16));
        }
    };
    auto issue_v = [&](const char* tile, int valid) {
        if (valid == 16) {
            issue_v_full(tile);
        } else {
            const char* p = tile + 4096 + c * 16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {  // raw piece r of this lane is part of token row 4r + g4
                const int row = 4 * r + g4 < valid ? 4 * r + g4 : 0;
                v[r].u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + row * 256));
            }
        }
    };
    char* scratch = lds + wave * kOpenScratch;
    const int n_full = min(wg->n_full[wave], wi.n_tiles);
    int t = 0;
    int meta = 16 << 20;
    if (F8 && n_full > 2) {
        // fp8 pools: a tile is half the bytes, so one tile in flight per wavefront is half the bytes in flight,
        // too little to keep the memory system busy.  The full tiles but the last go through a pipeline two
        // tiles deep: two sets of raw registers, A (k8, v8) and B, tile j of the pipeline in one of them by
        // turns, each refilled with tile j + 2 as soon as its codes have been widened.  The last full tile L is
        // left in flight in set A for the loop below, as the one-deep loop leaves it.
        if constexpr (F8) {
            const int L = n_full - 1;
            u32x4 k8b[2], v8b[2];
            float k8sb = 1.0f, v8sb = 1.0f;
            auto load_raw = [&](const char* tile, u32x4 (&kk)[2], u32x4 (&vv)[2], float& ks, float& vs, bool want_k, bool want_v) {
                const char* p = tile + lane * 16;
                if (want_k) {
#pragma unroll
                    for (int rp = 0; rp < 2; ++rp) kk[rp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + rp * 1024));
                    ks = *reinterpret_cast<const float*>(tile + kFp8ScaleOfs);
                }
                if (want_v) {
#pragma unroll
                    for (int rp = 0; rp < 2; ++rp)
                        vv[rp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + kFp8HalfBytes + rp * 1024));
                    vs = *reinterpret_cast<const float*>(tile + kFp8ScaleOfs + 4);
                }
            };
            // tile j, whose codes are in (kk, vv); then (refill): tile j + 2 into the same registers
            auto step = [&](int j, u32x4 (&kk)[2], u32x4 (&vv)[2], float& ks, float& vs, bool refill) {
                const int mt = mine[j].meta;
                const int lo = mt & 1023, hi = (mt >> 10) & 1023;
                const char* tn = refill ? head_base + mine[j + 2].blk * block_stride : nullptr;
                f32x4 sj[NT];
                fp8_operands(kk, ks, k);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (NT == 1 || touches(nt, lo, hi)) sj[nt] = products(k, st[nt]);
                if (refill) load_raw(tn, kk, vv, ks, vs, true, false);
                bool on[NT], in_range[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    on[nt] = NT == 1 || touches(nt, lo, hi);
                    in_range[nt] = my_j[nt] >= lo && my_j[nt] < hi;
                    if (on[nt] && (mt >> 30)) mask_tokens(sj[nt], visible(mt, my_j[nt] - lo), g4);
                }
                move_references<NT>(st, sj, on, in_range, scale_log2e);
                fp8_operands(vv, vs, v);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (on[nt]) weigh_values(v, st[nt], sj[nt], in_range[nt], scale_log2e);
                if (refill) load_raw(tn, kk, vv, ks, vs, false, true);
            };
            load_raw(head_base + mine[0].blk * block_stride, k8, v8, k8s, v8s, true, true);
            if (L & 1) {  // an odd number of tiles before the last: one of them alone, so that the rest go in pairs
                step(0, k8, v8, k8s, v8s, false);
                load_raw(head_base + mine[1].blk * block_stride, k8, v8, k8s, v8s, true, true);
                t = 1;
            }
            // L - t is even and at least 2: tiles t (in A) and t + 1 (into B) start the pairs
            load_raw(head_base + mine[t + 1].blk * block_stride, k8b, v8b, k8sb, v8sb, true, true);
            for (; t + 2 < L; t += 2) {
                step(t, k8, v8, k8s, v8s, true);
                step(t + 1, k8b, v8b, k8sb, v8sb, true);
            }
            step(t, k8, v8, k8s, v8s, true);          // refills A with tile L
            step(t + 1, k8b, v8b, k8sb, v8sb, false);
            t = L;
            meta = mine[L].meta;
        }
    } else if (n_full > 0) {
        // full tiles whose successor is full too: nothing but unconditional loads in this loop
        meta = mine[0].meta;
        const char* first = head_base + mine[0].blk * block_stride;
        issue_k_full(first);
        issue_v_full(first);
        for (; t + 1 < n_full; ++t) {
            const int lo = meta & 1023, hi = (meta >> 10) & 1023;
            const char* tn = head_base + mine[t + 1].blk * block_stride;
            const int meta_n = mine[t + 1].meta;
            f32x4 s[NT];
            k_ready(16);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (NT == 1 || touches(nt, lo, hi)) s[nt] = products(k, st[nt]);
            issue_k_full(tn);
            bool on[NT], in_range[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                on[nt] = NT == 1 || touches(nt, lo, hi);
                in_range[nt] = my_j[nt] >= lo && my_j[nt] < hi;
                if (on[nt] && (meta >> 30)) mask_tokens(s[nt], visible(meta, my_j[nt] - lo), g4);
            }
            move_references<NT>(st, s, on, in_range, scale_log2e);
            v_ready(16);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (on[nt]) weigh_values(v, st[nt], s[nt], in_range[nt], scale_log2e);
            issue_v_full(tn);
            meta = meta_n;
        }
    } else if (wi.n_tiles > 0) {
        meta = mine[0].meta;
        const char* first = head_base + mine[0].blk * block_stride;
        issue_k(first, (meta >> 20) & 31);
        issue_v(first, (meta >> 20) & 31);
    }
    // the last full tile and the open tiles
    for (; t < wi.n_tiles; ++t) {
        const bool more = t + 1 < wi.n_tiles;
        const int lo = meta & 1023, hi = (meta >> 10) & 1023, valid = (meta >> 20) & 31;
        const char* tn = nullptr;
        int meta_n = 16 << 20;
        if (more) {
            tn = head_base + mine[t + 1].blk * block_stride;
            meta_n = mine[t + 1].meta;
        }
        f32x4 s[NT];
        k_ready(valid);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (NT == 1 || touches(nt, lo, hi)) s[nt] = products(k, st[nt]);
        if (more) issue_k(tn, (meta_n >> 20) & 31);  // K registers are free again
        if (valid < 16) {
            // open block: its V half arrived row-major; turn it into operand order through LDS
#pragma unroll
            for (int r = 0; r < 4; ++r)
                *reinterpret_cast<u32x4*>(scratch + (4 * r + g4) * kOpenRowStride + c * 16) = v[r].u;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            v_operands_from_rows(scratch, kOpenRowStride, g4, c, v);
            __builtin_amdgcn_wave_barrier();
        }
        v_ready(valid);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (NT > 1 && !touches(nt, lo, hi)) continue;
            if (valid < 16 || (meta >> 30)) mask_tokens(s[nt], visible(meta, my_j[nt] - lo), g4);
            accumulate(v, st[nt], s[nt], my_j[nt] >= lo && my_j[nt] < hi, scale_log2e);
        }
        if (more) issue_v(tn, (meta_n >> 20) & 31);
        meta = meta_n;
    }

    // ---- results ------------------------------------------------------------------------------
    if (NT == 1 && (wi.flags & kWaveSplit)) {
        // the four wavefronts hold the same rows over different tiles: fold 1..3 into 0 through LDS
        RowState& s0 = st[0];
        float lt = s0.l;
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        float* so = reinterpret_cast<float*>(lds);           // [3][16 rows][128]
        float* sml = so + 3 * 16 * 128;                       // [3][16 rows][2]
        __syncthreads();  // every wavefront is done with its transpose scratch, which this area overlaps
        if (wave > 0) {
            float* dst = so + ((wave - 1) * 16 + c) * 128 + 4 * g4;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) *reinterpret_cast<f32x4*>(dst + 16 * jj) = s0.o[jj];
            if (g4 == 0) {
                sml[((wave - 1) * 16 + c) * 2] = s0.m;
                sml[((wave - 1) * 16 + c) * 2 + 1] = lt;
            }
        }
        __syncthreads();
        if (wave > 0) return;
        float mw[3], lw[3], mx = s0.m;
#pragma unroll
        for (int w2 = 0; w2 < 3; ++w2) {
            mw[w2] = sml[(w2 * 16 + c) * 2];
            lw[w2] = sml[(w2 * 16 + c) * 2 + 1];
            mx = fmaxf(mx, mw[w2]);
        }
        // a wavefront that saw no tile of a row left m = -inf and sums of zero for it
        const float a0 = (s0.m == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(s0.m - mx);
        lt *= a0;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) s0.o[jj] *= a0;
#pragma unroll
        for (int w2 = 0; w2 < 3; ++w2) {
            const float aw = (mw[w2] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw[w2] - mx);
            lt += aw * lw[w2];
            const float* src = so + (w2 * 16 + c) * 128 + 4 * g4;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) s0.o[jj] += aw * *reinterpret_cast<const f32x4*>(src + 16 * jj);
        }
        s0.m = mx;
        s0.l = g4 == 0 ? lt : 0.0f;  // back to one share per lane: the four lanes of a row add up to the sum
        __builtin_amdgcn_wave_barrier();
    }

    if ((wi.flags & kWaveDirect) && cand_mask != nullptr) {
        // Multi-candidate call: each thread's candidates are one more tile of at most 8 token rows
        // (row-major, a row every n_kv * 128 elements), visible to a row only where its mask bit is set.
        const int rank_lo = wi.grp_lo / n_sl, rank_hi = (wi.grp_lo + wi.n_grp - 1) / n_sl;
        const int64_t tok_stride = (int64_t)n_kv * 256;  // bytes between candidate rows of one kv head
        for (int ru = rank_lo; ru <= rank_hi; ++ru) {
            const int listed_u = plan.dfs_threads ? plan.dfs_threads[ru] : ru;
            const int64_t base = ((int64_t)listed_u * n_cand * n_kv + kvh) * 256;
            const char* kb = reinterpret_cast<const char*>(cand_k) + base;
            const char* vb = reinterpret_cast<const char*>(cand_v) + base;
            Frag kc[4], vc[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // rows past the last candidate: re-read candidate 0 (finite values under probability 0)
                kc[r].u = *reinterpret_cast<const u32x4*>(kb + (c < n_cand ? c : 0) * tok_stride + g4 * 64 + r * 16);
                const int row = 4 * r + g4 < n_cand ? 4 * r + g4 : 0;
                const u32x4 vr = *reinterpret_cast<const u32x4*>(vb + row * tok_stride + c * 16);
                *reinterpret_cast<u32x4*>(scratch + (4 * r + g4) * kOpenRowStride + c * 16) = vr;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            v_operands_from_rows(scratch, kOpenRowStride, g4, c, vc);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                uint32_t tm = 0;
                if (my_j[nt] != 0x7fff) {
                    const int grp = wi.grp_lo + my_j[nt];
                    const int rk = grp / n_sl, r2 = (grp - rk * n_sl) * rps + within;
                    if (rk == ru) tm = cand_mask[(int64_t)listed_u * n_cand + r2 / group];
                }
                if (__builtin_amdgcn_ballot_w64(tm != 0) == 0) continue;
                f32x4 sc = products(kc, st[nt]);
                mask_tokens(sc, tm, g4);
                accumulate(vc, st[nt], sc, tm != 0, scale_log2e);
            }
        }
    }

#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float lt = st[nt].l;
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (my_j[nt] == 0x7fff) continue;
        int rk, r2;
        int64_t qrow, slot;
        locate(nt, rk, r2, qrow, slot);
        if (wi.flags & kWaveDirect) {
            // the row's whole root path was covered here: normalise and write the output row
            const float inv = 1.0f / lt;
            uint16_t* dst = out + qrow * 128 + 4 * g4;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                u32x2 pk;
                pk.x = pack_bf16_pair(st[nt].o[jj][0] * inv, st[nt].o[jj][1] * inv);
                pk.y = pack_bf16_pair(st[nt].o[jj][2] * inv, st[nt].o[jj][3] * inv);
                __builtin_nontemporal_store(pk, reinterpret_cast<u32x2*>(dst + 16 * jj));
            }
        } else {
            // streaming stores: a partial result is read once, by the merge kernel
            float* dst = part.o + slot * 128 + 4 * g4;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                __builtin_nontemporal_store(st[nt].o[jj], reinterpret_cast<f32x4*>(dst + 16 * jj));
            if (g4 == 0) {
                __builtin_nontemporal_store(st[nt].m, part.ml + slot * 2);
                __builtin_nontemporal_store(lt, part.ml + slot * 2 + 1);
            }
        }
    }
}

}  // namespace

hipError_t launch_attention_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan, int n_cand,
                                 PartialBuf part, const void* cand_k, const void* cand_v, const uint8_t* mask,
                                 void* out, ClassStreams& cs, hipStream_t st) {
    // workgroups are sorted by class: [matrix units | 2 row tiles per wavefront | 1], heaviest first in each.
    // Matrix units go first, alone, on the caller's stream: their workgroups need 64 KB of LDS and most of a
    // SIMD's registers, and beside a kernel of small workgroups they wait until that kernel has drained
    // (measured: a 100 us launch took as long as the 800 us launch beside it).  Of the two row-tile classes
    // the last one present runs on the caller's stream and the other beside it on a side stream that waits
    // for the caller's stream first and that the caller's stream then waits for.
    int first[3], last = -1, n_present = 0;
    for (int cls = 0, f = 0; cls < 3; ++cls) {
        first[cls] = f;
        f += plan.n_wg_class[cls];
        if (cls > 0 && plan.n_wg_class[cls] > 0) last = cls, ++n_present;
        if ((int64_t)plan.n_wg_class[cls] * s.n_kv > 0x7fffffff) return hipErrorInvalidValue;
    }
    hipError_t e;
    if (plan.n_wg_class[0] > 0 &&
        (e = launch_attention_units_bf16(s, pool, q, plan, first[0], plan.n_wg_class[0], n_cand, part, st)) != hipSuccess)
        return e;
    if (last < 0) return hipSuccess;
    const bool side_by_side = n_present > 1 && !cs.serial;
    if (side_by_side) {
        if (!cs.fork) {
            if ((e = hipEventCreateWithFlags(&cs.fork, hipEventDisableTiming)) != hipSuccess) return e;
        }
        for (int k = 0; k < 2; ++k) {
            if (!cs.aux[k] && (e = hipStreamCreateWithFlags(&cs.aux[k], hipStreamNonBlocking)) != hipSuccess) return e;
            if (!cs.join[k] && (e = hipEventCreateWithFlags(&cs.join[k], hipEventDisableTiming)) != hipSuccess) return e;
        }
        if ((e = hipEventRecord(cs.fork, st)) != hipSuccess) return e;
    }
    int side = 0;
    bool used[2] = {false, false};
    for (int cls = 1; cls < 3; ++cls) {
        const int count = plan.n_wg_class[cls];
        if (count == 0) continue;
        hipStream_t on = st;
        if (cls != last && side_by_side) {
            on = cs.aux[side];
            if ((e = hipStreamWaitEvent(on, cs.fork, 0)) != hipSuccess) return e;
        }
        const unsigned n_wg = (unsigned)count * (unsigned)s.n_kv;
#define APAR_LAUNCH(NTV, F8V)                                                                                           \
    hipLaunchKernelGGL((attention_bf16<NTV, F8V>), dim3(n_wg), dim3(256), 0, on, (const char*)pool, (const uint16_t*)q, \
                       plan, first[cls], n_cand, s.n_q, s.n_kv, s.group, s.scale_log2e, part,                           \
                       (const uint16_t*)cand_k, (const uint16_t*)cand_v, mask, (uint16_t*)out)
        if (s.fp8_sealed) {
            if (cls == 1) APAR_LAUNCH(2, true);
            else APAR_LAUNCH(1, true);
        } else {
            if (cls == 1) APAR_LAUNCH(2, false);
            else APAR_LAUNCH(1, false);
        }
#undef APAR_LAUNCH
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (cls != last && side_by_side) {
            if ((e = hipEventRecord(cs.join[side], on)) != hipSuccess) return e;
            used[side] = true;
            ++side;
        }
    }
    for (int k = 0; k < 2; ++k)
        if (used[k] && (e = hipStreamWaitEvent(st, cs.join[k], 0)) != hipSuccess) return e;
    return hipSuccess;
}

}  // namespace apar
