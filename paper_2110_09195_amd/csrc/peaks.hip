// Measured-peak probes (see include/snn_peaks.h): the yardsticks of the roofline that bench.py
// reports.  Every kernel stays inside the buffers it is given and ends after a fixed trip count.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "snn_peaks.h"

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

inline int launched() { return hipGetLastError() == hipSuccess ? 0 : -4; }

// ---- HBM ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <bool NT>
__global__ __launch_bounds__(256) void fill_kernel(u32x4 *__restrict__ dst, size_t n16)
{
    // every block fills one contiguous piece (measured faster than pieces interleaved over the blocks: 5.3 against
    // 3.7 TB/s for non-temporal stores)
    const u32x4 v = {1u, 2u, 3u, (uint32_t)threadIdx.x};
    const size_t piece = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t end = (blockIdx.x + 1) * piece < n16 ? (blockIdx.x + 1) * piece : n16;
    for (size_t i = (size_t)blockIdx.x * piece + threadIdx.x; i < end; i += 256) {
        if (NT) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

// read-only stream: every block reads one contiguous piece (measured faster than pieces interleaved over the
// blocks: 7.1 against 5.9 TB/s with non-temporal loads), four 16-byte loads in flight per lane, folded into one
// word per lane
template <bool NT>
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *__restrict__ out)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    const size_t piece = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t first = (size_t)blockIdx.x * piece;
    const size_t end = first + piece < n16 ? first + piece : n16;
    size_t i = first + threadIdx.x;
    for (; i + 768 < end; i += 1024) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = NT ? __builtin_nontemporal_load(src + i + u * 256) : src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u];
    }
    for (; i < end; i += 256) acc ^= NT ? __builtin_nontemporal_load(src + i) : src[i];
    // one word per wave leaves (a word per lane would be 16 MB of writes in the read stream)
    uint32_t f = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) f ^= __shfl_xor(f, d);
    if ((threadIdx.x & 63) == 0) out[(size_t)blockIdx.x * 256 + threadIdx.x] = f;
}

// ---- integer VALU ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void valu_xor_bcnt_kernel(uint32_t *out, int iters)
{
    uint32_t x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0x9e3779b9u * (uint32_t)(i + 1) + threadIdx.x;
    uint32_t acc[4] = {0, 0, 0, 0};
    uint32_t w = blockIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i & 3] += __popc(x[i] ^ w);       // v_xor_b32 + v_bcnt_u32_b32 (with its addend)
        w = w * 1664525u + 1013904223u;                                     // wave-uniform
    }
    out[blockIdx.x * 256 + threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
}

// ---- matrix cores ---------------------------------------------------------------------------------
__device__ inline uint32_t mix(uint32_t v)
{
    v ^= v >> 16;
    v *= 0x7feb352du;
    v ^= v >> 15;
    v *= 0x846ca68bu;
    v ^= v >> 16;
    return v;
}

// FP6 e2m3 code of an integer in [-7, 7]
__device__ inline uint32_t fp6_code(int v)
{
    const uint32_t s = v < 0 ? 32u : 0u;
    const int a = v < 0 ? -v : v;
    const uint32_t mag = a == 0 ? 0u : a == 1 ? 8u : a < 4 ? 16u + 4u * (uint32_t)(a - 2) : 24u + 2u * (uint32_t)(a - 4);
    return s | mag;
}

__device__ inline void make_operands(int pattern, uint32_t lane_seed, v8i &a, v8i &b)
{
    uint32_t aw[8] = {0, 0, 0, 0, 0, 0, 0, 0}, bw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (pattern == 0) {
        for (int i = 0; i < 4; ++i) aw[i] = mix(lane_seed + 17u * i);
        for (int i = 0; i < 6; ++i) bw[i] = mix(lane_seed * 3u + 29u * i);
    } else if (pattern == 1) {
        const uint32_t k = mix(lane_seed) & 31u;                      // the member this (channel, channel) pair selects
        aw[k >> 3] = 2u << (4 * (k & 7u));                            // FP4 1.0 in slot k
        for (int j = 0; j < 32; ++j) {
            const uint32_t c = fp6_code((int)(mix(lane_seed + 101u * j) % 10u) - 4);
            const int bit = 6 * j;
            bw[bit >> 5] |= c << (bit & 31);
            if ((bit & 31) > 26) bw[(bit >> 5) + 1] |= c >> (32 - (bit & 31));
        }
    }
    a = (v8i){(int)aw[0], (int)aw[1], (int)aw[2], (int)aw[3], 0, 0, 0, 0};
    b = (v8i){(int)bw[0], (int)bw[1], (int)bw[2], (int)bw[3], (int)bw[4], (int)bw[5], 0, 0};
}

template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_f4f6_kernel(float *out, unsigned long long *clocks, int pattern, int iters)
{
    v8i a, b;
    make_operands(pattern, (uint32_t)(threadIdx.x & 63) * 2654435761u + 1u, a, b);
    float keep = 0.0f;
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    if constexpr (SHAPE == 0) {
        v16f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = (v16f){0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4 /* A: FP4 */, 2 /* B: FP6 e2m3 */, 0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) keep += acc[i][r];
    } else {
        v4f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = (v4f){0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc[i], 4, 2, 0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) keep += acc[i][r];
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    out[blockIdx.x * 256 + threadIdx.x] = keep;
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = c1 - c0;
        clocks[2 * blockIdx.x + 1] = r1 - r0;
    }
}

// ---- stage 2 as byte-parallel adds with a wave-uniform register index -------------------------------
// Register plan of the loop (fixed, because the vector-register index mode addresses registers by number):
//   v[32:63]    the 32 responses, 4 pixels per register as bytes
//   v[64:127]   byte accumulators of 64 output channels
//   v[128:255]  the same accumulators widened to 16 bits: v[128 + 2 c] pixels 0 and 2, v[129 + 2 c] pixels 1 and 3
//   s[36:99]    four buffers of 16 indices (one per dword), loaded three chunks ahead of their use
// In index mode (s_set_gpr_idx_on ..., SRC0) the first source of every vector instruction is
// v[number + M0[7:0]]; s_set_gpr_idx_idx replaces M0[7:0] with the low byte of a scalar register.
// One v_add_u32 therefore is four gather-adds and costs one scalar instruction beside it, which
// another wave of the SIMD hides.  28 additions of values <= 9 fit a byte; then the bytes are
// spread to the 16-bit accumulators (6 instructions per output channel).
__global__ __launch_bounds__(256, 2) void swar_gather_kernel(uint32_t *out, const uint32_t *idx, int n_groups)
{
    uint32_t result;
    asm volatile(
        // responses: value(k) = (7 k + 3) mod 10 in every byte
        ".set snn_i, 0\n"
        ".rept 32\n"
        "  v_mov_b32 v[32 + snn_i], 0x01010101 * ((7 * snn_i + 3) %% 10)\n"
        "  .set snn_i, snn_i + 1\n"
        ".endr\n"
        ".set snn_i, 0\n"
        ".rept 192\n"
        "  v_mov_b32 v[64 + snn_i], 0\n"
        "  .set snn_i, snn_i + 1\n"
        ".endr\n"
        "s_mov_b64 s[28:29], %[idx]\n"
        "s_mov_b32 s26, %[groups]\n"
        "s_mov_b32 s25, 0x00ff00ff\n"
        // the first three chunks of indices
        "s_load_dwordx16 s[36:51], s[28:29], 0\n"
        "s_load_dwordx16 s[52:67], s[28:29], 64\n"
        "s_load_dwordx16 s[68:83], s[28:29], 128\n"
        "s_add_u32 s28, s28, 192\n"
        "s_addc_u32 s29, s29, 0\n"
        "snn_group_%=:\n"
        "s_movk_i32 s27, 28\n"
        "s_set_gpr_idx_on s36, 1\n"                     // SRC0 relative
        "snn_ci_%=:\n"
        // four chunks of 16 output channels; chunk j reads buffer j, and the buffer of chunk j - 1 is
        // refilled with the chunk three ahead once every load issued before has landed
        ".set snn_c, 0\n"
        ".rept 4\n"
        "  s_waitcnt lgkmcnt(0)\n"
        "  s_load_dwordx16 s[36 + 16 * ((snn_c + 3) %% 4):51 + 16 * ((snn_c + 3) %% 4)], s[28:29], 0\n"
        "  s_add_u32 s28, s28, 64\n"
        "  s_addc_u32 s29, s29, 0\n"
        "  .set snn_i, 0\n"
        "  .rept 16\n"
        "    s_set_gpr_idx_idx s[36 + 16 * snn_c + snn_i]\n"
        "    v_add_u32 v[64 + 16 * snn_c + snn_i], v32, v[64 + 16 * snn_c + snn_i]\n"
        "    .set snn_i, snn_i + 1\n"
        "  .endr\n"
        "  .set snn_c, snn_c + 1\n"
        ".endr\n"
        "s_sub_u32 s27, s27, 1\n"
        "s_cmp_lg_u32 s27, 0\n"
        "s_cbranch_scc1 snn_ci_%=\n"
        "s_set_gpr_idx_off\n"
        // widen: 16-bit accumulators += bytes, bytes = 0
        ".set snn_i, 0\n"
        ".rept 64\n"
        "  v_and_b32 v30, s25, v[64 + snn_i]\n"
        "  v_lshrrev_b32 v31, 8, v[64 + snn_i]\n"
        "  v_add_u32 v[128 + 2 * snn_i], v[128 + 2 * snn_i], v30\n"
        "  v_and_b32 v31, s25, v31\n"
        "  v_mov_b32 v[64 + snn_i], 0\n"
        "  v_add_u32 v[129 + 2 * snn_i], v[129 + 2 * snn_i], v31\n"
        "  .set snn_i, snn_i + 1\n"
        ".endr\n"
        "s_sub_u32 s26, s26, 1\n"
        "s_cmp_lg_u32 s26, 0\n"
        "s_cbranch_scc1 snn_group_%=\n"
        "s_waitcnt lgkmcnt(0)\n"                        // the loads issued past the last chunk (inside the index array's padding)
        // checksum: sum of all 16-bit fields
        "v_mov_b32 %[res], 0\n"
        ".set snn_i, 0\n"
        ".rept 128\n"
        "  v_and_b32 v30, 0xffff, v[128 + snn_i]\n"
        "  v_lshrrev_b32 v31, 16, v[128 + snn_i]\n"
        "  v_add3_u32 %[res], %[res], v30, v31\n"
        "  .set snn_i, snn_i + 1\n"
        ".endr\n"
        : [res] "=&v"(result)
        : [idx] "s"(idx), [groups] "s"(n_groups)
        : "memory", "scc",
          "s25", "s26", "s27", "s28", "s29", "s36", "s37", "s38", "s39", "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47",
          "s48", "s49", "s50", "s51", "s52", "s53", "s54", "s55", "s56", "s57", "s58", "s59", "s60", "s61", "s62", "s63",
          "s64", "s65", "s66", "s67", "s68", "s69", "s70", "s71", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79",
          "s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95",
          "s96", "s97", "s98", "s99",
          "v30", "v31", "v32", "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45",
          "v46", "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57", "v58", "v59", "v60", "v61",
          "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71", "v72", "v73", "v74", "v75", "v76", "v77",
          "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", "v88", "v89", "v90", "v91", "v92", "v93",
          "v94", "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108",
          "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122",
          "v123", "v124", "v125", "v126", "v127", "v128", "v129", "v130", "v131", "v132", "v133", "v134", "v135", "v136",
          "v137", "v138", "v139", "v140", "v141", "v142", "v143", "v144", "v145", "v146", "v147", "v148", "v149", "v150",
          "v151", "v152", "v153", "v154", "v155", "v156", "v157", "v158", "v159", "v160", "v161", "v162", "v163", "v164",
          "v165", "v166", "v167", "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", "v176", "v177", "v178",
          "v179", "v180", "v181", "v182", "v183", "v184", "v185", "v186", "v187", "v188", "v189", "v190", "v191", "v192",
          "v193", "v194", "v195", "v196", "v197", "v198", "v199", "v200", "v201", "v202", "v203", "v204", "v205", "v206",
          "v207", "v208", "v209", "v210", "v211", "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", "v220",
          "v221", "v222", "v223", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", "v233", "v234",
          "v235", "v236", "v237", "v238", "v239", "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", "v248",
          "v249", "v250", "v251", "v252", "v253", "v254", "v255");
    out[blockIdx.x * 256 + threadIdx.x] = result;
}

}  // namespace

extern "C" {

int snn_peak_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes == 0 || bytes % 4096) return -1;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src, n16);
    return launched();
}

int snn_peak_fill(void *dst, size_t bytes, int nontemporal, void *stream)
{
    if (!dst || bytes == 0 || bytes % 4096) return -1;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    if (nontemporal) hipLaunchKernelGGL(fill_kernel<true>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, n16);
    else hipLaunchKernelGGL(fill_kernel<false>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, n16);
    return launched();
}

int snn_peak_read(const void *src, size_t bytes, int nontemporal, uint32_t *out, void *stream)
{
    if (!src || !out || bytes == 0 || bytes % 4096) return -1;
    const size_t n16 = bytes / 16;
    const unsigned blocks = SNN_PEAK_READ_BLOCKS;
    if (nontemporal) hipLaunchKernelGGL(read_kernel<true>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src, n16, out);
    else hipLaunchKernelGGL(read_kernel<false>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src, n16, out);
    return launched();
}

int snn_peak_valu_xor_bcnt(uint32_t *out, int iters, int blocks, void *stream)
{
    if (!out || iters < 1 || blocks < 1) return -1;
    hipLaunchKernelGGL(valu_xor_bcnt_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
    return launched();
}

size_t snn_peak_mfma_out_bytes(int blocks) { return blocks < 1 ? 0 : (size_t)blocks * (256 * 4 + 16); }

int snn_peak_mfma_f4f6(float *out, int shape, int pattern, int iters, int blocks, void *stream)
{
    if (!out || iters < 1 || blocks < 1 || shape < 0 || shape > 1 || pattern < 0 || pattern > 2) return -1;
    unsigned long long *clocks = (unsigned long long *)(out + (size_t)blocks * 256);
    if (shape == 0)
        hipLaunchKernelGGL(mfma_f4f6_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, clocks, pattern, iters);
    else
        hipLaunchKernelGGL(mfma_f4f6_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, clocks, pattern, iters);
    return launched();
}

int snn_peak_swar_gather(uint32_t *out, const uint32_t *idx, int n_ci, int blocks, void *stream)
{
    if (!out || !idx || n_ci < 28 || n_ci % 28 || n_ci > 7168 || blocks < 1) return -1;
    hipLaunchKernelGGL(swar_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, idx, n_ci / 28);
    return launched();
}

}  // extern "C"
