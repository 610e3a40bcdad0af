// Device-side bodies of the two small operations of a layer's forward pass (Alg. 1): sign +
// bit-packing of activations into packed rows, and the nearest-subset-member projection of
// real-valued kernels (Eq. 2 / Eq. 5).  Each is used by its own kernel and by the fused front
// kernel of snn_subbit_forward, which is what makes the two paths agree bit for bit.
#pragma once

#include "snn_internal.h"

namespace snn {

// Activations to pack are read exactly once, every byte of a cache line by one instruction: loaded
// non-temporally they stream past the caches instead of displacing what the next kernel reads.
// (Not so the kernels to project: a lane's nine loads touch the same lines again.)
__device__ inline float4 load_once4(const float *p)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 t = __builtin_nontemporal_load((const f32x4 *)p);
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ inline float load_once(const float *p) { return __builtin_nontemporal_load(p); }

// OR over the eight lanes 8 g .. 8 g + 7, valid in lane 8 g (all that the packing needs): two quad permutations
// and a shift by four lanes inside the row of sixteen, as data-parallel-primitive operands of the vector unit
// (the generic shuffle goes through the LDS pipeline with an address per lane).
__device__ inline uint32_t or_of_eight_lanes(uint32_t w)
{
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, true);
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x104 /* row_shl:4: lane i reads lane i + 4 */, 0xF, 0xF, true);
    return w;
}

constexpr int PACK_THREADS = 256;
constexpr int PACK_U = 2;                                  // 16-byte loads in flight per thread (2: 7 % faster than 4 on 51 MB inputs)
constexpr int PACK_CHUNK = PACK_THREADS * 4 * PACK_U;      // elements whose sign bits are staged in LDS per pass
constexpr int PACK_LDS_WORDS = PACK_CHUNK / 32 + 2;

// How launch_pack_rows cuts [rows][W] into blocks.
struct PackRowsPlan {
    int rows_per_block;      // whole rows per block (1 when a row is longer than PACK_CHUNK)
    int vec;                 // every block starts 16-byte aligned: 16-byte loads
    int64_t blocks;
};

inline PackRowsPlan pack_rows_plan(const float *x, int64_t rows, int W)
{
    PackRowsPlan pl;
    // whole rows per block, a multiple of four of them so that every block starts 16-byte aligned
    pl.rows_per_block = 1;
    if (W <= PACK_CHUNK) {
        pl.rows_per_block = PACK_CHUNK / W;
        if (pl.rows_per_block >= 4) pl.rows_per_block &= ~3;
    }
    const bool aligned_rows = ((int64_t)pl.rows_per_block * W) % 4 == 0 && (W <= PACK_CHUNK || W % 4 == 0);
    pl.vec = (((uintptr_t)x & 15) == 0 && aligned_rows) ? 1 : 0;
    pl.blocks = (rows + pl.rows_per_block - 1) / pl.rows_per_block;
    return pl;
}

// One block of PACK_THREADS threads packs rows [block * rows_per_block, ...) of x[rows][W].
// 16-byte loads -> four sign bits per lane -> eight lanes OR their nibbles into one word of a flat
// bit stream in LDS (`bits`, PACK_LDS_WORDS words) -> one output word per thread, cut out of the
// stream at the row's bit offset (rows need not be multiples of 32 wide).  `vec` says that every
// block's first element is 16-byte aligned; the last, partial group of four of a segment is read
// element by element.
__device__ inline void pack_rows_block(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t rows, int W,
                                       int WW, int rows_per_block, int vec, int64_t block, uint32_t *bits)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t r0 = block * rows_per_block;
    const int nrows = (int)min((int64_t)rows_per_block, rows - r0);
    if (nrows <= 0) return;

    // W <= PACK_CHUNK: one pass over nrows whole rows.  Otherwise rows_per_block == 1 and the
    // single row is cut into word-aligned segments of PACK_CHUNK elements.
    const int row_len = (W <= PACK_CHUNK) ? nrows * W : W;
    for (int seg = 0; seg < row_len; seg += PACK_CHUNK) {
        const int cnt = min(PACK_CHUNK, row_len - seg);
        const float *src = x + r0 * W + seg;
        float4 v[PACK_U];
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const int e = (u * PACK_THREADS + tid) * 4;
            if (vec && e + 3 < cnt) {
                v[u] = load_once4(src + e);
            } else {
                v[u].x = e < cnt ? src[e] : -1.0f;
                v[u].y = e + 1 < cnt ? src[e + 1] : -1.0f;
                v[u].z = e + 2 < cnt ? src[e + 2] : -1.0f;
                v[u].w = e + 3 < cnt ? src[e + 3] : -1.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const uint32_t nib = (v[u].x >= 0.0f ? 1u : 0u) | (v[u].y >= 0.0f ? 2u : 0u) | (v[u].z >= 0.0f ? 4u : 0u) |
                                 (v[u].w >= 0.0f ? 8u : 0u);
            uint32_t w = nib << (4 * (lane & 7));
            w = or_of_eight_lanes(w);
            if ((lane & 7) == 0) bits[(u * PACK_THREADS + tid) >> 3] = w;
        }
        __syncthreads();
        if (W <= PACK_CHUNK) {
            const int nwords = nrows * WW;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int rl = q / WW, j = q - rl * WW;
                const int o = rl * W + 32 * j;
                const int nb = min(32, W - 32 * j);
                const int sh = o & 31;
                uint32_t wv = bits[o >> 5] >> sh;
                if (sh + nb > 32) wv |= bits[(o >> 5) + 1] << (32 - sh);
                if (nb < 32) wv &= (1u << nb) - 1u;
                out[r0 * WW + q] = wv;
            }
        } else {
            const int nwords = (cnt + 31) >> 5;
            for (int q = tid; q < nwords; q += PACK_THREADS) {
                const int nb = min(32, cnt - 32 * q);
                uint32_t wv = bits[q];
                if (nb < 32) wv &= (1u << nb) - 1u;
                out[r0 * WW + (seg >> 5) + q] = wv;
            }
        }
        __syncthreads();
    }
}

// The same for blocks [b0, b1) of rows in one workgroup, as a stream: the loads of the next two blocks are in flight while
// the current one is packed, and the bit stream alternates between two LDS buffers (one barrier per block).  For
// rows that fit a pass (W <= PACK_CHUNK) whose blocks start 16-byte aligned (`vec`); `bits`: 2 x PACK_LDS_WORDS.
__device__ inline void pack_rows_stream(const float *__restrict__ x, uint32_t *__restrict__ out, int64_t rows, int W,
                                        int WW, int rows_per_block, int64_t b0, int64_t b1, uint32_t *bits)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    auto load_block = [&](int64_t b, float4 (&v)[PACK_U]) {
        const int64_t r0 = b * rows_per_block;
        const int cnt = (int)min((int64_t)rows_per_block, rows - r0) * W;
        const float *src = x + r0 * W;
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const int e = (u * PACK_THREADS + tid) * 4;
            if (e + 3 < cnt) {
                v[u] = load_once4(src + e);
            } else {
                v[u].x = e < cnt ? src[e] : -1.0f;
                v[u].y = e + 1 < cnt ? src[e + 1] : -1.0f;
                v[u].z = e + 2 < cnt ? src[e + 2] : -1.0f;
                v[u].w = e + 3 < cnt ? src[e + 3] : -1.0f;
            }
        }
    };
    float4 v[PACK_U], nx[PACK_U], nx2[PACK_U];
    if (b0 < b1) load_block(b0, v);
    if (b0 + 1 < b1) load_block(b0 + 1, nx);
    for (int64_t b = b0; b < b1; ++b) {
        if (b + 2 < b1) load_block(b + 2, nx2);
        uint32_t *bb = bits + (int)(b & 1) * PACK_LDS_WORDS;
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            const uint32_t nib = (v[u].x >= 0.0f ? 1u : 0u) | (v[u].y >= 0.0f ? 2u : 0u) | (v[u].z >= 0.0f ? 4u : 0u) |
                                 (v[u].w >= 0.0f ? 8u : 0u);
            uint32_t w = nib << (4 * (lane & 7));
            w = or_of_eight_lanes(w);
            if ((lane & 7) == 0) bb[(u * PACK_THREADS + tid) >> 3] = w;
        }
        __syncthreads();
        const int64_t r0 = b * rows_per_block;
        const int nwords = (int)min((int64_t)rows_per_block, rows - r0) * WW;
        for (int q = tid; q < nwords; q += PACK_THREADS) {
            const int rl = q / WW, j = q - rl * WW;
            const int o = rl * W + 32 * j;
            const int nb = min(32, W - 32 * j);
            const int sh = o & 31;
            uint32_t wv = bb[o >> 5] >> sh;
            if (sh + nb > 32) wv |= bb[(o >> 5) + 1] << (32 - sh);
            if (nb < 32) wv &= (1u << nb) - 1u;
            out[r0 * WW + q] = wv;
        }
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) {
            v[u] = nx[u];
            nx[u] = nx2[u];
        }
    }
}

// ---- projection ------------------------------------------------------------------------------------
// coef[K][12]: +1.0f / -1.0f for taps 0..8 of every subset member (+3 pad): three 16-byte reads
__device__ inline void project_fill_coef(float *coef, const uint16_t *__restrict__ codebook, int K, int tid, int nthreads)
{
    for (int i = tid; i < K * 12; i += nthreads) {
        const int k = i / 12, t = i - 12 * k;
        coef[i] = (t < 9 && ((codebook[k] >> (8 - t)) & 1)) ? 1.0f : -1.0f;
    }
}

// arg max_k <P_k, w> for Q kernels at once (one coefficient read serves the Q chains): the inner
// product is accumulated in fp32 from 0 over taps 0..8 in order, adding or subtracting w_t
// (fma(w_t, +-1, acc) rounds exactly like acc +- w_t); among equal scores the lowest index wins.
template <int Q>
__device__ inline void project_argmax(const float (&wt)[Q][9], const float *coef, int K, int (&best)[Q])
{
    float best_score[Q];
    auto score = [&](int k, float (&acc)[Q]) {
        const float4 ca = *(const float4 *)(coef + k * 12);          // wave-uniform address: broadcast
        const float4 cb = *(const float4 *)(coef + k * 12 + 4);
        const float c8 = coef[k * 12 + 8];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float a = 0.0f;
            a = __builtin_fmaf(wt[q][0], ca.x, a);
            a = __builtin_fmaf(wt[q][1], ca.y, a);
            a = __builtin_fmaf(wt[q][2], ca.z, a);
            a = __builtin_fmaf(wt[q][3], ca.w, a);
            a = __builtin_fmaf(wt[q][4], cb.x, a);
            a = __builtin_fmaf(wt[q][5], cb.y, a);
            a = __builtin_fmaf(wt[q][6], cb.z, a);
            a = __builtin_fmaf(wt[q][7], cb.w, a);
            a = __builtin_fmaf(wt[q][8], c8, a);
            acc[q] = a;
        }
    };
    // member 0 starts as the best (no test for "first member" inside the loop)
    score(0, best_score);
#pragma unroll
    for (int q = 0; q < Q; ++q) best[q] = 0;
    // unrolled so that the coefficient reads of several members are in flight and their chains interleave
#pragma unroll 4
    for (int k = 1; k < K; ++k) {
        float acc[Q];
        score(k, acc);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (acc[q] > best_score[q]) {
                best[q] = k;
                best_score[q] = acc[q];
            }
        }
    }
}

}  // namespace snn
