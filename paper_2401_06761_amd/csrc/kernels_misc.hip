// Row writes, copy-on-write block copies, row read-back, the fp32 attention
// kernel and the merge kernel (gfx950).
#include <hip/hip_runtime.h>

#include "apar_internal.hpp"

namespace apar {

namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// ---------------------------------------------------------------------------
// Row writes.  Row i of the call is taken from row src_rows[i] of k and v (from row
// i when src_rows is null).  bf16: 32 lanes per (row, kv head), eight pairs per
// workgroup; fp32: one wavefront per pair.
// bf16 pools keep a block that is still filling in plain row-major form (K rows
// then V rows, 256 contiguous bytes each), so an appended row is two full-line
// writes per half; seal_blocks_bf16 rewrites a block into matrix-core order once
// its sixteenth slot is written.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void append_rows_bf16(char* __restrict__ pool, const uint16_t* __restrict__ k,
                                                        const uint16_t* __restrict__ v,
                                                        const int32_t* __restrict__ codes,
                                                        const int32_t* __restrict__ src_rows, int n_rows, int n_kv,
                                                        int64_t tile_bytes) {
    const int64_t pair = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);  // (row, kv head), heads fastest
    const int lane = threadIdx.x & 31;
    if (pair >= (int64_t)n_rows * n_kv) return;
    const int row = (int)(pair / n_kv), h = (int)(pair - (int64_t)row * n_kv);
    const int32_t code = codes[row];
    const int slot = code & 15;
    char* tile = pool + ((int64_t)(code >> 4) * n_kv + h) * tile_bytes;
    const int64_t from = src_rows ? src_rows[row] : row;
    const uint16_t* src = (lane < 16 ? k : v) + (from * n_kv + h) * 128 + (lane & 15) * 8;
    *reinterpret_cast<uint4*>(tile + (lane < 16 ? 0 : 4096) + slot * 256 + (lane & 15) * 16) =
        *reinterpret_cast<const uint4*>(src);
}

// In-place row-major -> matrix-core order for blocks that just became full.
// One workgroup per (block, kv head): the 8 KiB tile goes through LDS.
__global__ __launch_bounds__(256) void seal_blocks_bf16(char* __restrict__ pool, const int32_t* __restrict__ blocks,
                                                        int n_kv, int64_t tile_bytes) {
    __shared__ __attribute__((aligned(16))) char raw[8192];
    const int t = threadIdx.x;
    char* tile = pool + ((int64_t)blocks[blockIdx.x] * n_kv + blockIdx.y) * tile_bytes;
    reinterpret_cast<uint4*>(raw)[t] = reinterpret_cast<const uint4*>(tile)[t];
    reinterpret_cast<uint4*>(raw)[256 + t] = reinterpret_cast<const uint4*>(tile)[256 + t];
    __syncthreads();
    // piece t of either half sits at byte t*16 of the half: load index r = t / 64, lane = t % 64
    const int r = t >> 6, lane = t & 63, g = lane >> 4, c = lane & 15;
    // K piece: K[token c][dims 32g + 8r .. +8]
    const uint4 kp = *reinterpret_cast<const uint4*>(raw + c * 256 + (32 * g + 8 * r) * 2);
    // V piece: V[tokens 4g..4g+3][dim 32r + c], then V[tokens 4g..4g+3][dim 32r + 16 + c]
    const uint16_t* vr = reinterpret_cast<const uint16_t*>(raw + 4096);
    uint32_t w[4];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int dim = 32 * r + 16 * hh + c;
        w[2 * hh] = (uint32_t)vr[(4 * g + 0) * 128 + dim] | ((uint32_t)vr[(4 * g + 1) * 128 + dim] << 16);
        w[2 * hh + 1] = (uint32_t)vr[(4 * g + 2) * 128 + dim] | ((uint32_t)vr[(4 * g + 3) * 128 + dim] << 16);
    }
    reinterpret_cast<uint4*>(tile)[t] = kp;
    reinterpret_cast<uint4*>(tile)[256 + t] = make_uint4(w[0], w[1], w[2], w[3]);
}

// fp8 pools: a block that just became full is rewritten from bf16 rows into fp8 codes in matrix-core order,
// with one power-of-two scale for its K half and one for its V half: the smallest power of two s for which
// max |x| / s <= 448, the largest e4m3 magnitude (1 if the half is all zeros), so that the codes use the top
// binade of the format.  Codes are rounded to nearest even by the hardware conversion.  One workgroup per
// (block, kv head); the 8 KiB of rows go through LDS.
__device__ __forceinline__ float fp8_scale_for(float amax) {
    if (!(amax > 0.0f) || !(amax < INFINITY)) return 1.0f;
    int k;
    const float f = frexpf(amax, &k);            // amax = f * 2^k, f in [0.5, 1); 448 = 0.875 * 2^9
    const int e = (f <= 0.875f) ? k - 9 : k - 8;
    return ldexpf(1.0f, e < -126 ? -126 : e);
}

__global__ __launch_bounds__(256) void seal_blocks_fp8(char* __restrict__ pool, const int32_t* __restrict__ blocks,
                                                       int n_kv, int64_t tile_bytes) {
    __shared__ __attribute__((aligned(16))) char raw[8192];
    __shared__ float wave_max[2][4];
    const int t = threadIdx.x;
    char* tile = pool + ((int64_t)blocks[blockIdx.x] * n_kv + blockIdx.y) * tile_bytes;
    const uint4 a = reinterpret_cast<const uint4*>(tile)[t], b = reinterpret_cast<const uint4*>(tile)[256 + t];
    reinterpret_cast<uint4*>(raw)[t] = a;
    reinterpret_cast<uint4*>(raw)[256 + t] = b;
    // largest magnitude of either half (thread t holds 8 K elements in a and 8 V elements in b)
    float mk = 0.0f, mv = 0.0f;
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        mk = fmaxf(mk, fmaxf(fabsf(__uint_as_float(aw[i] << 16)), fabsf(__uint_as_float(aw[i] & 0xffff0000u))));
        mv = fmaxf(mv, fmaxf(fabsf(__uint_as_float(bw[i] << 16)), fabsf(__uint_as_float(bw[i] & 0xffff0000u))));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        mk = fmaxf(mk, __shfl_xor(mk, o, 64));
        mv = fmaxf(mv, __shfl_xor(mv, o, 64));
    }
    if ((t & 63) == 0) wave_max[0][t >> 6] = mk, wave_max[1][t >> 6] = mv;
    __syncthreads();
    const float ks = fp8_scale_for(fmaxf(fmaxf(wave_max[0][0], wave_max[0][1]), fmaxf(wave_max[0][2], wave_max[0][3])));
    const float vs = fp8_scale_for(fmaxf(fmaxf(wave_max[1][0], wave_max[1][1]), fmaxf(wave_max[1][2], wave_max[1][3])));
    const float kinv = 1.0f / ks, vinv = 1.0f / vs;  // powers of two: exact
    // thread t writes the 8 bytes of piece r of lane `lane` of each half: r = t / 64
    const int r = t >> 6, lane = t & 63, g = lane >> 4, c = lane & 15;
    const uint16_t* kr = reinterpret_cast<const uint16_t*>(raw) + c * 128 + 32 * g + 8 * r;  // K[token c][dims 32g + 8r ..]
    const uint16_t* vr = reinterpret_cast<const uint16_t*>(raw + 4096);
    float kx[8], vx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) kx[i] = bf16_to_f32(kr[i]) * kinv;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int i = 0; i < 4; ++i) vx[4 * hh + i] = bf16_to_f32(vr[(4 * g + i) * 128 + 32 * r + 16 * hh + c]) * vinv;
    uint32_t kw[2], vw[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        kw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(kx[4 * w], kx[4 * w + 1], 0, false);
        kw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(kx[4 * w + 2], kx[4 * w + 3], kw[w], true);
        vw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(vx[4 * w], vx[4 * w + 1], 0, false);
        vw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(vx[4 * w + 2], vx[4 * w + 3], vw[w], true);
    }
    const int ofs = (r >> 1) * 1024 + lane * 16 + (r & 1) * 8;
    *reinterpret_cast<uint2*>(tile + ofs) = make_uint2(kw[0], kw[1]);
    *reinterpret_cast<uint2*>(tile + kFp8HalfBytes + ofs) = make_uint2(vw[0], vw[1]);
    if (t == 0) *reinterpret_cast<float2*>(tile + kFp8ScaleOfs) = make_float2(ks, vs);
}

__global__ __launch_bounds__(64) void append_rows_f32(char* __restrict__ pool, const float* __restrict__ k,
                                                      const float* __restrict__ v, const int32_t* __restrict__ codes,
                                                      const int32_t* __restrict__ src_rows, int n_kv, int d,
                                                      int64_t tile_bytes) {
    const int row = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int32_t code = codes[row];
    const int slot = code & 15;
    float* tile = reinterpret_cast<float*>(pool + ((int64_t)(code >> 4) * n_kv + h) * tile_bytes);
    const int64_t from = src_rows ? src_rows[row] : row;
    const float* ksrc = k + (from * n_kv + h) * d;
    const float* vsrc = v + (from * n_kv + h) * d;
    for (int x = lane; x < d; x += 64) {
        tile[slot * d + x] = ksrc[x];
        tile[16 * d + slot * d + x] = vsrc[x];
    }
}

__global__ __launch_bounds__(64) void read_rows_bf16(const char* __restrict__ pool, uint16_t* __restrict__ k,
                                                     uint16_t* __restrict__ v, const int32_t* __restrict__ codes,
                                                     int n_kv, int64_t tile_bytes, int fp8_sealed) {
    const int row = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int32_t code = codes[row];
    const bool sealed = (code & kCodeSealed) != 0;  // the row's block is full, hence in matrix-core order
    const int slot = code & 15;
    const char* tile = pool + ((int64_t)((code & ~kCodeSealed) >> 4) * n_kv + h) * tile_bytes;
    uint16_t* kdst = k + ((int64_t)row * n_kv + h) * 128;
    uint16_t* vdst = v + ((int64_t)row * n_kv + h) * 128;
    if (sealed && fp8_sealed) {  // fp8 codes times the half's power-of-two scale: exact in bf16
        const float2 sc = *reinterpret_cast<const float2*>(tile + kFp8ScaleOfs);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int dim = lane + 64 * e;
            const uint32_t kc = *reinterpret_cast<const uint8_t*>(tile + fp8_k_offset(slot, dim));
            const uint32_t vc = *reinterpret_cast<const uint8_t*>(tile + kFp8HalfBytes + fp8_v_offset(slot, dim));
            kdst[dim] = f32_to_bf16_rne(__builtin_amdgcn_cvt_f32_fp8(kc, 0) * sc.x);
            vdst[dim] = f32_to_bf16_rne(__builtin_amdgcn_cvt_f32_fp8(vc, 0) * sc.y);
        }
        return;
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int dim = lane + 64 * e;
        const int ko = sealed ? bf16_k_offset(slot, dim) : slot * 256 + dim * 2;
        const int vo = sealed ? bf16_v_offset(slot, dim) : slot * 256 + dim * 2;
        kdst[dim] = *reinterpret_cast<const uint16_t*>(tile + ko);
        vdst[dim] = *reinterpret_cast<const uint16_t*>(tile + 4096 + vo);
    }
}

__global__ __launch_bounds__(64) void read_rows_f32(const char* __restrict__ pool, float* __restrict__ k,
                                                    float* __restrict__ v, const int32_t* __restrict__ codes,
                                                    int n_kv, int d, int64_t tile_bytes) {
    const int row = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int32_t code = codes[row];
    const int slot = code & 15;
    const float* tile = reinterpret_cast<const float*>(pool + ((int64_t)(code >> 4) * n_kv + h) * tile_bytes);
    for (int x = lane; x < d; x += 64) {
        k[((int64_t)row * n_kv + h) * d + x] = tile[slot * d + x];
        v[((int64_t)row * n_kv + h) * d + x] = tile[16 * d + slot * d + x];
    }
}

// Copy-on-write: whole blocks, 16 bytes per lane.  grid = (pairs, slices).
__global__ __launch_bounds__(256) void copy_blocks(char* __restrict__ pool, const int32_t* __restrict__ pairs,
                                                   int64_t block_bytes) {
    const int32_t src = pairs[2 * blockIdx.x], dst = pairs[2 * blockIdx.x + 1];
    const uint4* s = reinterpret_cast<const uint4*>(pool + (int64_t)src * block_bytes);
    uint4* d = reinterpret_cast<uint4*>(pool + (int64_t)dst * block_bytes);
    const int64_t n16 = block_bytes / 16;
    for (int64_t i = (int64_t)blockIdx.y * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.y * blockDim.x)
        d[i] = s[i];
}

// ---------------------------------------------------------------------------
// fp32 attention: one wavefront per query row, plain vector arithmetic, row-major
// tiles.  Used by fp32 pools, where results must hold to 1e-5 and the matrix
// cores' bf16 inputs would not.  Follows the same plan as the bf16 kernel: row c
// of wavefront k of a workgroup walks the group's shared tiles and wavefront k's
// own tiles and takes those whose row-group range contains its own.
// grid = (plan workgroups, kv heads, 4 wavefronts x 4 row tiles x 16 rows); block = 64 lanes over the head dim.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attention_f32(const char* __restrict__ pool, const float* __restrict__ q,
                                                    PlanDev plan, int n_cand, int n_q, int n_kv, int group,
                                                    float scale_log2e, int64_t tile_bytes, PartialBuf part,
                                                    const float* __restrict__ cand_k,
                                                    const float* __restrict__ cand_v,
                                                    const uint8_t* __restrict__ cand_mask,
                                                    float* __restrict__ out) {
    constexpr int E = D / 64;
    const int lane = threadIdx.x;
    const int kvh = blockIdx.y;
    // row c of row tile nt of wavefront `wave`: tile nt holds row groups nt * cap .. of the wavefront
    const int wave = blockIdx.z >> 6, nt = (blockIdx.z >> 4) & 3, c = blockIdx.z & 15;
    const WgDesc* wg = plan.wgs + blockIdx.x;
    if (nt >= (wg->row_tiles & 255)) return;
    const WaveItem wi = wg->w[wave];
    const int rps = plan.rows_per_slice, n_sl = plan.n_slices, rpt = plan.rows_per_thread;
    const int cap = 16 / rps, jc = c / rps, within = c - jc * rps;
    const int j = nt * cap + jc;
    const int grp = wi.grp_lo + j;
    const int rank = grp / n_sl, rr = (grp - rank * n_sl) * rps + within;
    if (jc >= cap || j >= wi.n_grp || rr >= rpt) return;
    const int listed = plan.dfs_threads ? plan.dfs_threads[rank] : rank;
    const int cc = rr / group, hq = kvh * group + (rr - cc * group);
    const int64_t qrow = ((int64_t)listed * n_cand + cc) * n_q + hq;
    float qv[E], acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) qv[e] = q[qrow * D + lane + 64 * e], acc[e] = 0.0f;
    float m = -INFINITY, l = 0.0f;
    // a split group's four wavefront items hold the same rows and a quarter of the tiles each
    const bool split = (wi.flags & kWaveSplit) != 0;
    if (split && wave != 0) return;
    const int n_lists = split ? 5 : 2;
    for (int list = 0; list < n_lists; ++list) {
        const WaveItem& src = wg->w[list < 2 ? wave : list - 1];
        const TileRef* tiles = plan.tiles + (list == 0 ? wg->coop_ofs : src.tile_ofs);
        const int n_tiles = list == 0 ? wg->n_coop : src.n_tiles;
        const int my_j = list == 0 ? j + (wi.grp_lo - wg->grp_base) : j;
        for (int t = 0; t < n_tiles; ++t) {
            const int meta = tiles[t].meta;
            const int lo = meta & 1023, hi = (meta >> 10) & 1023;
            if (my_j < lo || my_j >= hi) continue;
            // a causal tile (bit 30) shows its first row group `first` slots (bits 25-29), every further one one more
            int valid = (meta >> 20) & 31;
            if (meta >> 30) valid = min(valid, ((meta >> 25) & 31) + (my_j - lo));
            const float* tile = reinterpret_cast<const float*>(pool + ((int64_t)tiles[t].blk * n_kv + kvh) * tile_bytes);
            for (int tok = 0; tok < valid; ++tok) {
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < E; ++e) dot += qv[e] * tile[tok * D + lane + 64 * e];
                const float sc = wave_sum(dot) * scale_log2e;
                const float m_new = fmaxf(m, sc);
                const float alpha = exp2f(m - m_new), pr = exp2f(sc - m_new);
                l = l * alpha + pr;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = acc[e] * alpha + pr * tile[16 * D + tok * D + lane + 64 * e];
                m = m_new;
            }
        }
    }
    if (wi.flags & kWaveDirect) {
        if (cand_mask != nullptr) {  // multi-candidate call: the candidates this row may see
            const uint32_t bits = cand_mask[(int64_t)listed * n_cand + cc];
            for (int cp = 0; cp < n_cand; ++cp) {
                if (!((bits >> cp) & 1u)) continue;
                const int64_t base = (((int64_t)listed * n_cand + cp) * n_kv + kvh) * D;
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < E; ++e) dot += qv[e] * cand_k[base + lane + 64 * e];
                const float sc = wave_sum(dot) * scale_log2e;
                const float m_new = fmaxf(m, sc);
                const float alpha = exp2f(m - m_new), pr = exp2f(sc - m_new);
                l = l * alpha + pr;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = acc[e] * alpha + pr * cand_v[base + lane + 64 * e];
                m = m_new;
            }
        }
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < E; ++e) out[qrow * D + lane + 64 * e] = acc[e] * inv;
        return;
    }
    const int64_t slot = ((int64_t)(wi.part_base + rank - wi.grp_lo / n_sl) * n_cand + cc) * n_q + hq;
#pragma unroll
    for (int e = 0; e < E; ++e) part.o[slot * D + lane + 64 * e] = acc[e];
    if (lane == 0) {
        part.ml[slot * 2] = m;
        part.ml[slot * 2 + 1] = l;
    }
}

// ---------------------------------------------------------------------------
// Merge: sixteen lanes per (listed thread, candidate, q head).  Folds the partial
// results on the thread's root path (log-sum-exp in base 2), adds the candidate
// keys the mask lets this candidate see, normalises and writes the output row.
// Threads without partial results were already written by the attention kernel.
// ---------------------------------------------------------------------------
// E consecutive elements starting at element idx (a multiple of E) as floats: 16-byte loads.
template <int E, bool BF16>
__device__ __forceinline__ void load_run(const void* base, int64_t idx, float (&x)[E]) {
    if constexpr (BF16) {
        static_assert(E == 8, "a bf16 run is one 16-byte load");
        const uint4 u = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + idx);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] = __uint_as_float(w[e] << 16);
            x[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            const float4 f = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + idx + e);
            x[e] = f.x, x[e + 1] = f.y, x[e + 2] = f.z, x[e + 3] = f.w;
        }
    }
}

__device__ __forceinline__ float sum_over_16_lanes(float x) {
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// A workgroup takes 16 consecutive q heads of one (listed thread, candidate): sixteen lanes per output
// row, each with D / 16 consecutive dims, so the four rows of a wavefront read 4 * D consecutive floats
// of every partial result in one go.
template <int D, bool BF16>
__global__ __launch_bounds__(256) void merge_rows(PlanDev plan, PartialBuf part, const void* __restrict__ qv,
                                                  const void* __restrict__ ckv, const void* __restrict__ cvv,
                                                  const uint8_t* __restrict__ mask, int n_cand, int n_q, int n_kv,
                                                  int group, float scale_log2e, void* __restrict__ outv) {
    constexpr int E = D / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c16 = lane & 15;
    const int head = blockIdx.x * 16 + wave * 4 + (lane >> 4);
    const int c = blockIdx.y, i = blockIdx.z;
    const int p0 = plan.path_ofs[i], p1 = plan.path_ofs[i + 1];
    if (p0 == p1) return;  // the attention kernel wrote this thread's rows itself (candidates included)
    const bool ok = head < n_q;
    const int hq = ok ? head : 0;  // rows past the last head redo head 0 and write nothing
    float m = -INFINITY;
    for (int p = p0; p < p1; ++p) {
        const int64_t slot = ((int64_t)plan.path_ids[p] * n_cand + c) * n_q + hq;
        m = fmaxf(m, part.ml[slot * 2]);
    }
    // logits of the visible candidates
    float cs[8];
    uint32_t bits = 0;
    if (mask != nullptr) {
        bits = mask[(int64_t)i * n_cand + c];
        float qr[E];
        load_run<E, BF16>(qv, (((int64_t)i * n_cand + c) * n_q + hq) * D + c16 * E, qr);
        for (int cp = 0; cp < n_cand; ++cp) {
            cs[cp] = -INFINITY;
            if ((bits >> cp) & 1u) {
                float kr[E];
                load_run<E, BF16>(ckv, (((int64_t)i * n_cand + cp) * n_kv + hq / group) * D + c16 * E, kr);
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < E; ++e) dot += qr[e] * kr[e];
                cs[cp] = sum_over_16_lanes(dot) * scale_log2e;
                m = fmaxf(m, cs[cp]);
            }
        }
    }
    float l = 0.0f, acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.0f;
#pragma unroll 2
    for (int p = p0; p < p1; ++p) {
        const int64_t slot = ((int64_t)plan.path_ids[p] * n_cand + c) * n_q + hq;
        const float2 ml = *reinterpret_cast<const float2*>(part.ml + slot * 2);
        float o[E];
        load_run<E, false>(part.o, slot * D + c16 * E, o);
        const float w = exp2f(ml.x - m);
        l += w * ml.y;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] += w * o[e];
    }
    if (mask != nullptr) {
        for (int cp = 0; cp < n_cand; ++cp) {
            if ((bits >> cp) & 1u) {
                const float w = exp2f(cs[cp] - m);
                float vr[E];
                load_run<E, BF16>(cvv, (((int64_t)i * n_cand + cp) * n_kv + hq / group) * D + c16 * E, vr);
                l += w;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] += w * vr[e];
            }
        }
    }
    if (!ok) return;
    const float inv = 1.0f / l;
    const int64_t obase = (((int64_t)i * n_cand + c) * n_q + hq) * D + c16 * E;
    if constexpr (BF16) {
        uint32_t w[E / 2];
#pragma unroll
        for (int e = 0; e < E / 2; ++e)
            w[e] = (uint32_t)f32_to_bf16_rne(acc[2 * e] * inv) | ((uint32_t)f32_to_bf16_rne(acc[2 * e + 1] * inv) << 16);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(outv) + obase) = uint4{w[0], w[1], w[2], w[3]};
    } else {
#pragma unroll
        for (int e = 0; e < E; e += 4)
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(outv) + obase + e) =
                float4{acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv};
    }
}

}  // namespace

hipError_t launch_attention_bf16(const Shape& s, const void* pool, const void* q, const PlanDev& plan, int n_cand,
                                 PartialBuf part, const void* cand_k, const void* cand_v, const uint8_t* mask,
                                 void* out, ClassStreams& cs, hipStream_t st);

// ---------------------------------------------------------------------------
// Fixed workspace of apar_decode_attention_fixed: the plan tables and the partial results of one call live
// in this array instead of in memory the library allocates.  Every GPU the library runs on holds its own
// copy of the array, at its own address, until the process ends.  In host code the array's name is only a
// handle of the symbol, not a device address: the address comes from hipGetSymbolAddress, once per device
// with that device current, and that pointer is what kernels and copies are given.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[(size_t)APAR_FIXED_PLAN_BYTES + (size_t)APAR_FIXED_PARTIAL_BYTES];

namespace {
constexpr int kMaxDevices = 64;
char* g_scratch_ptr[kMaxDevices] = {};  // per device: where its copy of `scratch` lives (null: not asked yet)
}  // namespace

hipError_t fixed_workspace_of_device(int device, char** out) {
    if (device < 0 || device >= kMaxDevices || !out) return hipErrorInvalidValue;
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr || ((uintptr_t)ptr & 255)) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = (char*)ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

hipError_t launch_append_rows(const Shape& s, void* pool, const void* k, const void* v, const int32_t* dst_codes,
                              const int32_t* src_rows, int n_rows, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    // grid.x carries the rows: go through them in slices that fit the grid limits
    const int kMaxRows = 1 << 20;
    for (int r0 = 0; r0 < n_rows; r0 += kMaxRows) {
        const int nr = n_rows - r0 < kMaxRows ? n_rows - r0 : kMaxRows;
        dim3 grid(nr, s.n_kv);
        // with a source index the rows are addressed from the arrays' start; without, slice by slice
        const int64_t row_elems = src_rows ? 0 : (int64_t)s.n_kv * s.d;
        const int32_t* from = src_rows ? src_rows + r0 : nullptr;
        if (s.dtype == APAR_BF16) {
            const unsigned n_wg = (unsigned)(((int64_t)nr * s.n_kv + 7) / 8);
            hipLaunchKernelGGL(append_rows_bf16, dim3(n_wg), dim3(256), 0, st, (char*)pool,
                               (const uint16_t*)k + r0 * row_elems, (const uint16_t*)v + r0 * row_elems,
                               dst_codes + r0, from, nr, s.n_kv, s.tile_bytes);
        } else {
            hipLaunchKernelGGL(append_rows_f32, grid, dim3(64), 0, st, (char*)pool, (const float*)k + r0 * row_elems,
                               (const float*)v + r0 * row_elems, dst_codes + r0, from, s.n_kv, s.d, s.tile_bytes);
        }
    }
    return hipGetLastError();
}

hipError_t launch_seal_blocks(const Shape& s, void* pool, const int32_t* blocks, int n_blocks, hipStream_t st) {
    if (n_blocks <= 0 || s.dtype != APAR_BF16) return hipSuccess;
    const int kSlice = 1 << 20;
    for (int b0 = 0; b0 < n_blocks; b0 += kSlice) {
        const int nb = n_blocks - b0 < kSlice ? n_blocks - b0 : kSlice;
        if (s.fp8_sealed)
            hipLaunchKernelGGL(seal_blocks_fp8, dim3(nb, s.n_kv), dim3(256), 0, st, (char*)pool, blocks + b0, s.n_kv,
                               s.tile_bytes);
        else
            hipLaunchKernelGGL(seal_blocks_bf16, dim3(nb, s.n_kv), dim3(256), 0, st, (char*)pool, blocks + b0, s.n_kv,
                               s.tile_bytes);
    }
    return hipGetLastError();
}

hipError_t launch_block_copies(const Shape& s, void* pool, const int32_t* pairs, int n_pairs, hipStream_t st) {
    if (n_pairs <= 0) return hipSuccess;
    int slices = (int)((s.block_bytes / 16 + 255) / 256);
    if (slices > 64) slices = 64;
    if (slices < 1) slices = 1;
    hipLaunchKernelGGL(copy_blocks, dim3(n_pairs, slices), dim3(256), 0, st, (char*)pool, pairs, s.block_bytes);
    return hipGetLastError();
}

// words[pairs[2 i]] = pairs[2 i + 1]: brings staged plan tables up to date word by word.  Pairs that name the
// same word carry the same value.
__global__ __launch_bounds__(256) void scatter_words(int32_t* __restrict__ words, const int32_t* __restrict__ pairs, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int2 p = reinterpret_cast<const int2*>(pairs)[i];
    words[p.x] = p.y;
}

hipError_t launch_scatter_words(int32_t* words, const int32_t* pairs, int n_pairs, hipStream_t st) {
    if (n_pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(scatter_words, dim3((n_pairs + 255) / 256), dim3(256), 0, st, words, pairs, n_pairs);
    return hipGetLastError();
}

hipError_t launch_read_rows(const Shape& s, const void* pool, const int32_t* src_codes, int n_rows, void* k_out,
                            void* v_out, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    dim3 grid(n_rows, s.n_kv);
    if (s.dtype == APAR_BF16)
        hipLaunchKernelGGL(read_rows_bf16, grid, dim3(64), 0, st, (const char*)pool, (uint16_t*)k_out,
                           (uint16_t*)v_out, src_codes, s.n_kv, s.tile_bytes, s.fp8_sealed);
    else
        hipLaunchKernelGGL(read_rows_f32, grid, dim3(64), 0, st, (const char*)pool, (float*)k_out, (float*)v_out,
                           src_codes, s.n_kv, s.d, s.tile_bytes);
    return hipGetLastError();
}

hipError_t launch_attention_partial(const Shape& s, const void* pool, const void* q, const PlanDev& plan, int n_cand,
                                    PartialBuf part, const void* cand_k, const void* cand_v, const uint8_t* mask,
                                    void* out, ClassStreams& cs, hipStream_t st) {
    if (plan.n_wg <= 0) return hipSuccess;
    if (s.dtype == APAR_BF16)
        return launch_attention_bf16(s, pool, q, plan, n_cand, part, cand_k, cand_v, mask, out, cs, st);
    dim3 grid(plan.n_wg, s.n_kv, 256);
    if (s.d == 64)
        hipLaunchKernelGGL(attention_f32<64>, grid, dim3(64), 0, st, (const char*)pool, (const float*)q, plan, n_cand,
                           s.n_q, s.n_kv, s.group, s.scale_log2e, s.tile_bytes, part, (const float*)cand_k,
                           (const float*)cand_v, mask, (float*)out);
    else
        hipLaunchKernelGGL(attention_f32<128>, grid, dim3(64), 0, st, (const char*)pool, (const float*)q, plan, n_cand,
                           s.n_q, s.n_kv, s.group, s.scale_log2e, s.tile_bytes, part, (const float*)cand_k,
                           (const float*)cand_v, mask, (float*)out);
    return hipGetLastError();
}

hipError_t launch_merge(const Shape& s, const PlanDev& plan, PartialBuf part, const void* q, const void* cand_k,
                        const void* cand_v, const uint8_t* mask, int n_cand, void* out, hipStream_t st) {
    if (plan.n_threads <= 0) return hipSuccess;
    // grid.z carries the listed threads (limit 65535): go through them in slices
    const int kSlice = 32768;
    for (int i0 = 0; i0 < plan.n_threads; i0 += kSlice) {
        const int ni = plan.n_threads - i0 < kSlice ? plan.n_threads - i0 : kSlice;
        PlanDev pl = plan;
        pl.path_ofs = plan.path_ofs + i0;
        const int64_t e = s.dtype == APAR_F32 ? 4 : 2;
        const int64_t qofs = (int64_t)i0 * n_cand * s.n_q * s.d * e;
        const int64_t kofs = (int64_t)i0 * n_cand * s.n_kv * s.d * e;
        const void* q2 = (const char*)q + qofs;
        const void* ck2 = cand_k ? (const char*)cand_k + kofs : nullptr;
        const void* cv2 = cand_v ? (const char*)cand_v + kofs : nullptr;
        const uint8_t* mk2 = mask ? mask + (int64_t)i0 * n_cand : nullptr;
        void* out2 = (char*)out + qofs;
        dim3 grid((s.n_q + 15) / 16, n_cand, ni);
#define APAR_MERGE(DD, BF)                                                                                        \
    hipLaunchKernelGGL((merge_rows<DD, BF>), grid, dim3(256), 0, st, pl, part, q2, ck2, cv2, mk2, n_cand, s.n_q, \
                       s.n_kv, s.group, s.scale_log2e, out2)
        if (s.dtype == APAR_BF16) APAR_MERGE(128, true);
        else if (s.d == 64) APAR_MERGE(64, false);
        else APAR_MERGE(128, false);
#undef APAR_MERGE
    }
    return hipGetLastError();
}

}  // namespace apar
