// The sub-bit convolution of Sec. 4.5 / Fig. 6 on gfx950, +-1 activations (SNN_ACT_BIN_ROWS).
//
// Stage 1 (each input channel x each of the K subset kernels) and stage 2 (per output channel,
// gather the responses its indices select and sum them along c_in) run fused in one kernel; the
// K x c_in response maps never leave the chip.
//
//   A workgroup owns a tile of TP = 16*G consecutive output pixels and a block of output
//   channels.  Per chunk of CIC input channels it builds, in LDS, the table T[ci][k][pixel] of
//   MATCH COUNTS (0..9, one byte per pixel, so four pixels share a 32-bit word); every lane then
//   gathers 16-byte rows T[ci][idx[co][ci]][16 pixels] (ds_read_b128) and adds them with plain
//   32-bit adds, one v_add3_u32 accumulating four pixels of two input channels.  Bytes are widened
//   into 16-bit pairs every <= 28 input channels (28 * 9 = 252 < 256).  The response of a kernel
//   is 2 * matches - taps, so
//       S = 2 * (M - corr[co][type]) - C_in * valid_taps(type)
//   where M is the accumulated match count and corr removes the matches that taps outside the
//   image (read as bit 0) fake; it depends only on the output channel and the pixel's border type.
//
//   Stage 1 for K <= 64 is a table lookup: the 9-bit window of a pixel indexes a 512-entry LDS
//   table of K match counts, and a 4x4 byte transpose (v_perm_b32) turns four pixels' rows into
//   the pixel-packed words of T.  The loop is software-pipelined: windows of chunk c+2 are
//   fetched from HBM/L2 while chunk c+1 is looked up and chunk c is gathered, with one barrier
//   per chunk.  For K > 64 (only the full 512-kernel set, used as a cross-check of the 1-bit
//   kernel) a plain XOR + popcount kernel is used instead.
//
// The kernel is bound by LDS bandwidth (one byte read per (pixel, c_out, c_in)), not by HBM.
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include "subbit_common.h"

namespace snn {

namespace {

constexpr int SB_WIDEN = 28;         // input channels a byte accumulator can take (28 * 9 <= 255)
constexpr int SB_LUT_MAXK = 64;
constexpr int SB_TPAD = 64;          // bytes between the T tables of two input channels (bank spread)

struct SbParams {
    const uint32_t *x;
    const uint32_t *codes;    // [512] window-order codes
    const uint4 *lut;         // table image for the lookup kernel: [513][KP + 16] bytes (row 512 zero)
    const uint16_t *offs;     // [nchunks][COP][CIC] row byte offsets (idx * TP)
    const int32_t *corr;      // [COP][16]
    const float *alpha;
    float *y;
    Geom g;
    int COP;
    int nchunks;
    int vec4;                 // rows of 4 output pixels can be stored as float4
};

// ---- index preparation -------------------------------------------------------------------------
// One launch, three jobs (by block range):
//   offs[cc][co][cl] = min(idx[co][cc*CIC+cl], K-1) * row_bytes      (0 for padding)
//   corr[co][type]   = sum over c_in of the zero bits of the selected code at the taps that
//                      border type `type` puts outside the image
//   codes[k]         = code k in window order (tap t at bit t)
//   lut[window][k]   = 9 - popcount(window ^ code_k) as bytes, rows of KP + 16 bytes (an odd
//                      number of 16-byte pieces, which spreads random rows over the LDS banks),
//                      0 for k >= K, plus an all-zero row 512; copied to LDS by every workgroup
__global__ __launch_bounds__(256)
void subbit_prep_kernel(const uint16_t *__restrict__ codebook, const uint16_t *__restrict__ idx, int C_in,
                        int C_out, int COP, int K, int CIC, int nchunks, int row_bytes, int offs_blocks,
                        int lut_blocks, uint32_t *__restrict__ codes, uint16_t *__restrict__ offs,
                        int32_t *__restrict__ corr, uint32_t *__restrict__ lut)
{
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= (int)gridDim.x - lut_blocks) {
        // one thread per table word (four k)
        const int KP = (K + 15) & ~15;
        const int wpr = (KP + 16) / 4;                     // words per row
        const int i = ((int)blockIdx.x - ((int)gridDim.x - lut_blocks)) * 256 + tid;
        if (i < 513 * wpr) {
            const int win = i / wpr, kq = i - win * wpr;
            uint32_t word = 0;
            if (win < 512)
                for (int b = 0; b < 4; ++b) {
                    const int k = 4 * kq + b;
                    if (k < K) word |= (9u - __popc((uint32_t)win ^ code_to_window_order(codebook[k] & 511u))) << (8 * b);
                }
            lut[i] = word;
        }
        return;
    }
    if ((int)blockIdx.x < offs_blocks) {
        const int64_t gid = (int64_t)blockIdx.x * 256 + tid;
        const int64_t n_offs = (int64_t)nchunks * COP * CIC;
        if (gid < n_offs) {
            const int cl = (int)(gid % CIC);
            const int co = (int)((gid / CIC) % COP);
            const int cc = (int)(gid / ((int64_t)CIC * COP));
            const int ci = cc * CIC + cl;
            int k = 0;
            if (co < C_out && ci < C_in) k = min((int)idx[(int64_t)co * C_in + ci], K - 1);
            offs[gid] = (uint16_t)(k * row_bytes);
        }
        return;
    }
    const int b = blockIdx.x - offs_blocks;
    const int co = b * 4 + (tid >> 6);          // one wave per output channel
    const int lane = tid & 63;
    if (b == 0)
        for (int k = tid; k < 512; k += 256) codes[k] = k < K ? code_to_window_order(codebook[k] & 511u) : 0u;
    if (co >= COP) return;
    int zeros[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) zeros[t] = 0;
    if (co < C_out)
        for (int c0 = 0; c0 < C_in; c0 += 64) {
            const int ci = c0 + lane;
            uint32_t z = 0;
            if (ci < C_in) {
                const int k = min((int)idx[(int64_t)co * C_in + ci], K - 1);
                z = ~code_to_window_order(codebook[k] & 511u) & 511u;
            }
#pragma unroll
            for (int t = 0; t < 9; ++t) zeros[t] += __popcll(__ballot((z >> t) & 1u));
        }
    if (lane < 16) {
        const uint32_t inv = border_invalid_window(lane);
        int s = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((inv >> t) & 1u) s += zeros[t];
        corr[co * 16 + lane] = s;
    }
}

// ---- table-lookup kernel (K <= 64) -----------------------------------------------------------------

// base + low / high 16 bits of `packed` in one VALU operation (SDWA operand select).
__device__ inline uint32_t add_lo16(uint32_t packed, uint32_t base)
{
    uint32_t r;
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:DWORD"
        : "=v"(r) : "v"(packed), "v"(base));
    return r;
}
__device__ inline uint32_t add_hi16(uint32_t packed, uint32_t base)
{
    uint32_t r;
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:DWORD"
        : "=v"(r) : "v"(packed), "v"(base));
    return r;
}

// Window geometry of one pixel, arranged so that a window costs three funnel shifts:
//   bits(dy) = alignbit(row[jhi] & mhi[dy], row[jlo] & mlo[dy], sh) & 7
// Rows outside the image have both masks 0; the left border uses (hi = word 0, lo = 0, sh = 31);
// columns right of the image read the zero bits the packed layout guarantees.
// Window geometry, arranged so that the bits of a window row cost one funnel shift:
//   bits(dy) = alignbit(word_hi & mhi[dy], word_lo & mlo[dy], sh)
// starts at input column c0 = first window column - 1.  Rows outside the image have both masks
// 0; at the left border (c0 = -1) the pair is (hi = word 0, lo = 0, sh = 31); columns right of
// the image read the zero bits the packed layout guarantees.  Offsets are in bytes from x, for
// input channel 0.
struct WinGeom {
    uint32_t off_lo[3], off_hi[3];
    int sh;
    uint32_t mlo[3], mhi[3];
};

// (n, ho, wo): first output pixel whose window starts at this geometry (one pixel, or an aligned
// group of four pixels of one output row).
__device__ inline WinGeom win_geom_at(int n, int ho, int wo, const Geom &g)
{
    WinGeom q;
    const int hc = ho * g.stride, wc = wo * g.stride;
    const uint32_t plane0 = (uint32_t)n * (uint32_t)g.C_in * (uint32_t)(g.H * g.WW);
    const int c = wc - 1;
    int jlo, jhi;
    uint32_t ml, mh;
    if (c >= 0) {
        jlo = c >> 5;
        q.sh = c & 31;
        ml = ~0u;
        const bool has_hi = jlo + 1 < g.WW;
        jhi = has_hi ? jlo + 1 : jlo;
        mh = has_hi ? ~0u : 0u;
    } else {
        jlo = 0;
        jhi = 0;
        q.sh = 31;
        ml = 0u;
        mh = ~0u;
    }
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const int h = hc + dy - 1;
        const bool ok = h >= 0 && h < g.H;
        const uint32_t rowoff = plane0 + (uint32_t)((ok ? h : 0) * g.WW);
        q.off_lo[dy] = (rowoff + jlo) * 4u;
        q.off_hi[dy] = (rowoff + jhi) * 4u;
        q.mlo[dy] = ok ? ml : 0u;
        q.mhi[dy] = ok ? mh : 0u;
    }
    return q;
}

__device__ inline WinGeom win_geom(int64_t p, const Geom &g)
{
    if (p >= g.P) p = g.P - 1;
    const int n = (int)(p / g.HoWo);
    const int r = (int)(p - (int64_t)n * g.HoWo);
    const int ho = r / g.Wo;
    return win_geom_at(n, ho, r - ho * g.Wo, g);
}

struct WinRaw {
    uint32_t lo[3], hi[3];
};

// W1: packed rows are one word wide, so the "next word" is the same word and is not loaded again.
template <bool W1>
__device__ inline WinRaw win_load(const uint32_t *__restrict__ x, const WinGeom &q, uint32_t ci_bytes)
{
    WinRaw r;
    const char *xb = (const char *)x;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        r.lo[dy] = *(const uint32_t *)(xb + (size_t)(q.off_lo[dy] + ci_bytes));
        r.hi[dy] = W1 ? r.lo[dy] : *(const uint32_t *)(xb + (size_t)(q.off_hi[dy] + ci_bytes));
    }
    return r;
}

// the three window rows as bit strings starting at column c0
__device__ inline void win_rows(const WinRaw &r, const WinGeom &q, uint32_t row[3])
{
#pragma unroll
    for (int dy = 0; dy < 3; ++dy)
        row[dy] = __builtin_amdgcn_alignbit(r.hi[dy] & q.mhi[dy], r.lo[dy] & q.mlo[dy], q.sh);
}

// 9-bit window whose columns start `shift` bits into the row strings
__device__ inline uint32_t win_pick(const uint32_t row[3], int shift)
{
    return ((row[0] >> shift) & 7u) | (((row[1] >> shift) & 7u) << 3) | (((row[2] >> shift) & 7u) << 6);
}

// QUAD: W_out is a multiple of 4, so every aligned group of four tile pixels lies in one output
// row and stage 1 cuts its four windows out of three funnel-shifted row strings.  Otherwise the
// windows are extracted one pixel at a time and staged through LDS.
// MODE: 0 = windows one pixel at a time; 1 = the same with one-word rows; 2 = QUAD; 3 = QUAD with
// one-word rows.
template <int G, int J, int NW, int KP, int CIC, int MODE>
__global__ __launch_bounds__(NW * 64)
void subbit_lut_kernel(const SbParams p)
{
    constexpr bool QUAD = MODE >= 2;
    constexpr bool W1 = (MODE & 1) != 0;
    constexpr int NT = NW * 64;
    constexpr int TP = 16 * G;                     // pixels per tile
    constexpr int WPT = 4 * G;                     // 4-pixel words per tile row
    constexpr int CL = 64 / G;                     // output channels per wave instruction
    constexpr int COW = CL * J;                    // output channels per wave
    constexpr int KV = KP / 16;                    // 16-byte pieces per table row
    constexpr int LROW = KP + 16;                  // table row stride: an odd number of 16-byte pieces
    constexpr int TS = KP * TP + SB_TPAD;          // bytes per input channel in T
    constexpr int WM = QUAD ? 1 : (CIC * TP + NT - 1) / NT;      // per-pixel window items per thread and chunk
    constexpr int ITEMS = CIC * WPT;               // stage-1 items per chunk: (input channel, 4-pixel word)
    constexpr int SM = (ITEMS + NT - 1) / NT;
    constexpr int WCH = SB_WIDEN / CIC;            // chunks between widenings
    static_assert(NT % TP == 0 && NT % WPT == 0, "a thread keeps its pixels across items");
    static_assert(CIC == 4 || CIC == 8, "offsets of a chunk are one 8- or 16-byte load");

    const Geom &g = p.g;

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *lut = smem;                                        // [513][LROW]; row 512 is all zero
    unsigned char *Tbuf = lut + 513 * LROW;                           // [2][CIC][TS]
    uint16_t *wbuf = (uint16_t *)(Tbuf + 2 * CIC * TS);               // [2][CIC][TP]   (!QUAD only)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * TP;
    const int gq = lane % G, cl = lane / G;
    const int lane_co = blockIdx.y * (COW * NW) + wave * COW + cl * J;   // first of this lane's J channels
    const uint32_t plane_bytes = (uint32_t)(g.H * g.WW) * 4u;
    const int sstep = g.stride;

    // the table image was built once by the preparation kernel; copy it into LDS
    for (int i = tid; i < 513 * LROW / 16; i += NT) ((uint4 *)lut)[i] = p.lut[i];

    // ---- windows ------------------------------------------------------------------------------------
    // QUAD : this thread's stage-1 items all use pixel group (tid % WPT); their row words are
    //        fetched one chunk ahead into qraw.
    // !QUAD: this thread extracts pixel (tid % TP) for input channels tid / TP + m * (NT / TP); raw
    //        words are fetched two chunks ahead and the windows staged in wbuf.
    const WinGeom geo = win_geom(QUAD ? p_tile + 4 * (tid % WPT) : p_tile + (tid % TP), g);
    WinRaw qraw[QUAD ? SM : 1];
    uint32_t qok = 0;
    WinRaw raw[WM];
    uint32_t raw_ok = 0;                    // bit m: the item's input channel exists

    auto load_quads = [&](int chunk) {
        qok = 0;
#pragma unroll
        for (int m = 0; m < SM; ++m) {
            const int ci_l = (tid + m * NT) / WPT;
            const int ci = chunk * CIC + (ci_l < CIC ? ci_l : 0);
            qok |= (ci < g.C_in ? 1u : 0u) << m;
            qraw[m] = win_load<W1>(p.x, geo, (uint32_t)min(ci, g.C_in - 1) * plane_bytes);   // always a valid address
        }
    };
    auto load_windows = [&](int chunk) {
        raw_ok = 0;
#pragma unroll
        for (int m = 0; m < WM; ++m) {
            const int ci_l = tid / TP + m * (NT / TP);
            const int ci = chunk * CIC + (ci_l < CIC ? ci_l : 0);
            raw_ok |= (ci < g.C_in ? 1u : 0u) << m;
            raw[m] = win_load<W1>(p.x, geo, (uint32_t)min(ci, g.C_in - 1) * plane_bytes);
        }
    };
    // input channels past C_in get window 512, the all-zero table row
    auto store_windows = [&](int buf) {
#pragma unroll
        for (int m = 0; m < WM; ++m) {
            const int ci_l = tid / TP + m * (NT / TP);
            uint32_t row[3];
            win_rows(raw[m], geo, row);
            const uint32_t w = ((raw_ok >> m) & 1u) ? win_pick(row, 0) : 512u;
            if (ci_l < CIC) wbuf[(buf * CIC + ci_l) * TP + (tid % TP)] = (uint16_t)w;
        }
    };

    // stage 1 of one chunk: four windows -> four table rows -> transposed into T
    auto stage1 = [&](int buf) {
#pragma unroll
        for (int m = 0; m < SM; ++m) {
            const int it = tid + m * NT;
            if (ITEMS % NT != 0 && it >= ITEMS) break;
            const int wd = it % WPT;
            const int ci_l = it / WPT;
            const int pos = (wd % G) * 4 + wd / G;      // lane gq later reads words 4*gq .. 4*gq+3
            uint32_t w0, w1, w2, w3;
            if constexpr (QUAD) {
                uint32_t row[3];
                win_rows(qraw[m], geo, row);
                const bool ok = (qok >> m) & 1u;
                w0 = ok ? win_pick(row, 0) : 512u;
                w1 = ok ? win_pick(row, sstep) : 512u;
                w2 = ok ? win_pick(row, 2 * sstep) : 512u;
                w3 = ok ? win_pick(row, 3 * sstep) : 512u;
            } else {
                const uint2 w4 = *(const uint2 *)(wbuf + (buf * CIC + ci_l) * TP + 4 * wd);
                w0 = w4.x & 0xffffu;
                w1 = w4.x >> 16;
                w2 = w4.y & 0xffffu;
                w3 = w4.y >> 16;
            }
            const unsigned char *r0 = lut + w0 * LROW, *r1 = lut + w1 * LROW;
            const unsigned char *r2 = lut + w2 * LROW, *r3 = lut + w3 * LROW;
            uint32_t *Tw = (uint32_t *)(Tbuf + (buf * CIC + ci_l) * TS) + pos;
#pragma unroll
            for (int kv = 0; kv < KV; ++kv) {
                const uint4 v0 = *(const uint4 *)(r0 + kv * 16);
                const uint4 v1 = *(const uint4 *)(r1 + kv * 16);
                const uint4 v2 = *(const uint4 *)(r2 + kv * 16);
                const uint4 v3 = *(const uint4 *)(r3 + kv * 16);
                uint32_t o[16];
                transpose4x4(v0.x, v1.x, v2.x, v3.x, o + 0);
                transpose4x4(v0.y, v1.y, v2.y, v3.y, o + 4);
                transpose4x4(v0.z, v1.z, v2.z, v3.z, o + 8);
                transpose4x4(v0.w, v1.w, v2.w, v3.w, o + 12);
#pragma unroll
                for (int i = 0; i < 16; ++i) Tw[(kv * 16 + i) * WPT] = o[i];
            }
        }
    };

    uint32_t acc[J][4];
    uint32_t wide_e[J][4], wide_o[J][4];     // even / odd bytes of acc, as 16-bit pairs
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = wide_e[j][w] = wide_o[j][w] = 0;

    // offsets of a chunk: CIC u16 per output channel, contiguous
    typedef typename std::conditional<CIC == 8, uint4, uint2>::type offs_t;
    offs_t oa[J], ob[J];
    const offs_t *obase = (const offs_t *)p.offs + lane_co;
    auto load_offs = [&](int chunk, offs_t dst[J]) {
#pragma unroll
        for (int j = 0; j < J; ++j) dst[j] = obase[(int64_t)chunk * p.COP + j];
    };

    // ---- prologue ------------------------------------------------------------------------------
    load_offs(0, oa);
    if constexpr (QUAD) {
        load_quads(0);
        __syncthreads();                    // table visible
        stage1(0);
        load_quads(1);
    } else {
        load_windows(0);
        store_windows(0);
        load_windows(1);
        __syncthreads();                    // table and windows of chunk 0 visible
        stage1(0);
        store_windows(1);
        load_windows(2);
    }
    __syncthreads();

    int since_widen = 0;
    // one chunk: look up chunk c+1, gather chunk c (offsets in ocur), fetch the windows further ahead
    auto iteration = [&](int c, int buf, const offs_t ocur[J], offs_t onext[J]) {
        const bool more = c + 1 < p.nchunks;
        load_offs(more ? c + 1 : c, onext);
        if (more) stage1(buf ^ 1);
        if constexpr (QUAD) load_quads(c + 2);

        if (since_widen == WCH) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
                    wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
                    acc[j][w] = 0;
                }
            since_widen = 0;
        }
        ++since_widen;
        const uint32_t lb = (uint32_t)(buf * CIC * TS + gq * 16);
#pragma unroll
        for (int j = 0; j < J; ++j) {
            uint32_t ow[CIC / 2];
            ow[0] = ocur[j].x;
            ow[1] = ocur[j].y;
            if constexpr (CIC == 8) {
                ow[2] = ocur[j].z;
                ow[3] = ocur[j].w;
            }
#pragma unroll
            for (int q = 0; q < CIC / 2; ++q) {
                const uint4 va = *(const uint4 *)(Tbuf + add_lo16(ow[q], lb) + (2 * q) * TS);
                const uint4 vb = *(const uint4 *)(Tbuf + add_hi16(ow[q], lb) + (2 * q + 1) * TS);
                acc[j][0] = acc[j][0] + va.x + vb.x;
                acc[j][1] = acc[j][1] + va.y + vb.y;
                acc[j][2] = acc[j][2] + va.z + vb.z;
                acc[j][3] = acc[j][3] + va.w + vb.w;
            }
            // Finish this channel set's adds before the next set's gathers are issued: hoisting
            // all gathers pins 16 registers each and costs more occupancy than it hides latency.
            asm volatile("" : "+v"(acc[j][0]), "+v"(acc[j][1]), "+v"(acc[j][2]), "+v"(acc[j][3]) : : "memory");
        }

        if constexpr (!QUAD) {
            // windows of chunk c+2 (loaded one iteration ago) -> LDS; fetch chunk c+3
            store_windows(buf);
            load_windows(c + 3);
        }
        __syncthreads();
    };
    for (int c = 0; c < p.nchunks; c += 2) {
        iteration(c, 0, oa, ob);
        if (c + 1 < p.nchunks) iteration(c + 1, 1, ob, oa);
    }

    // ---- epilogue: S = 2 * (M - corr) - C_in * valid_taps, y = float(S) * alpha ---------------------
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
            wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
        }
    float a[J];
#pragma unroll
    for (int j = 0; j < J; ++j) a[j] = lane_co + j < g.C_out ? p.alpha[lane_co + j] : 0.0f;

#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // accumulator word w of lane gq holds tile pixels 4 * (w * G + gq) .. + 3
        const int64_t p0 = p_tile + 4 * (w * G + gq);
        if (p0 >= g.P) continue;
        int n = (int)(p0 / g.HoWo);
        int r = (int)(p0 - (int64_t)n * g.HoWo);
        int ho = r / g.Wo, wo = r - ho * g.Wo;
        float out[J][4];
        int rr[4], nn[4];
        bool ok[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            ok[b] = p0 + b < g.P;
            rr[b] = r;
            nn[b] = n;
            const int type = border_type(ho, wo, g.H, g.W, g.stride);
            const int base = border_valid_taps(type) * g.C_in;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                const int co = lane_co + j;
                const int cr = (type != 0 && co < g.C_out) ? p.corr[co * 16 + type] : 0;
                out[j][b] = (float)(2 * (M - cr) - base) * a[j];
            }
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) ho = 0;
            }
            if (++r == g.HoWo) {
                r = 0;
                ++n;
            }
        }
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int co = lane_co + j;
            if (co >= g.C_out) continue;
            if (p.vec4 && ok[3]) {
                float4 *dst = (float4 *)(p.y + ((int64_t)nn[0] * g.C_out + co) * g.HoWo + rr[0]);
                *dst = make_float4(out[j][0], out[j][1], out[j][2], out[j][3]);
            } else {
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (ok[b]) p.y[((int64_t)nn[b] * g.C_out + co) * g.HoWo + rr[b]] = out[j][b];
            }
        }
    }
}

// ---- wave-private variant of the table-lookup kernel ------------------------------------------------
// For layers with many output pixels.  Every wave owns a tile of 16 pixels and its own T table in
// LDS (lanes = 64 output channels, J sets of them), so stage 1 and stage 2 alternate inside the
// wave with no workgroup barrier; the workgroup only shares the 512-entry lookup table.  Waves
// progress independently, which hides the LDS and memory latencies that a barrier per chunk exposes.

constexpr int WV_NW = 8;       // waves per workgroup
constexpr int WV_CIC = 8;      // input channels per chunk

template <int J, int KP, int MODE>
__global__ __launch_bounds__(WV_NW * 64)
void subbit_wave_kernel(const SbParams p)
{
    constexpr bool QUAD = MODE >= 2;
    constexpr bool W1 = (MODE & 1) != 0;
    constexpr int NT = WV_NW * 64;
    constexpr int CIC = WV_CIC;
    constexpr int KV = KP / 16;
    constexpr int LROW = KP + 16;
    constexpr int TS = KP * 16 + 16;               // bytes per input channel in T: rows of 16 pixels, +16 spreads banks
    constexpr int ITEMS = CIC * 4 * KV;            // stage-1 items per chunk: (input channel, table piece, 4-pixel word)
    constexpr int SM = (ITEMS + 63) / 64;
    constexpr int WM = QUAD ? 1 : 2;               // per-pixel window items per lane: 16 pixels x 8 channels / 64
    constexpr int WCH = SB_WIDEN / CIC;

    const Geom &g = p.g;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *lut = smem;                                            // [513][LROW]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);            // scalar: per-tile geometry stays on the SALU
    unsigned char *T = lut + 513 * LROW + wave * (CIC * TS + CIC * 16 * 2);   // this wave's [CIC][TS]
    uint16_t *wbuf = (uint16_t *)(T + CIC * TS);                          // this wave's [CIC][16] windows (!QUAD)

    const int lane_co = blockIdx.y * (64 * J) + lane * J;
    const uint32_t plane_bytes = (uint32_t)(g.H * g.WW) * 4u;
    const int sstep = g.stride;

    for (int i = tid; i < 513 * LROW / 16; i += NT) ((uint4 *)lut)[i] = p.lut[i];

    __syncthreads();                              // lookup table visible; the only workgroup barrier

    // Persistent waves: wave (blockIdx.x, wave) takes 16-pixel tiles first, first + stride, ...
    const int64_t ntiles = (g.P + 15) / 16;
    const int64_t tstride = (int64_t)gridDim.x * WV_NW;
    for (int64_t tile = (int64_t)blockIdx.x * WV_NW + wave; tile < ntiles; tile += tstride) {
    const int64_t p_tile = tile * 16;
    // coordinates of the tile's first pixel (wave-uniform, scalar divisions)
    const int t_n = (int)(p_tile / g.HoWo);
    const int t_r = (int)(p_tile - (int64_t)t_n * g.HoWo);
    const int t_ho = t_r / g.Wo, t_wo = t_r - t_ho * g.Wo;

    // stage-1 item m of this lane: it = lane + 64 m -> wd = it % 4, kv = (it / 4) % KV, ci_l = it / (4 KV)
    // QUAD: all items of the lane share the pixel group wd = lane % 4.
    // The lane's pixel is at most 15 past the tile's first one: with rows of 16 or more pixels that
    // is at most one row (and one image) further, otherwise fall back to dividing.
    WinGeom geo;
    {
        const int d = QUAD ? 4 * (lane & 3) : (lane & 15);
        if (g.Wo >= 16) {
            int n = t_n, ho = t_ho, wo = t_wo + d;
            if (wo >= g.Wo) {
                wo -= g.Wo;
                if (++ho == g.Ho) {
                    ho = 0;
                    ++n;
                }
            }
            if (n >= g.N) {          // past the last pixel: any valid pixel will do, nothing is stored
                n = g.N - 1;
                ho = 0;
                wo = 0;
            }
            geo = win_geom_at(n, ho, wo, g);
        } else {
            geo = win_geom(p_tile + d, g);
        }
    }
    WinRaw qraw[QUAD ? SM : 1];
    uint32_t qok = 0;
    WinRaw raw[WM];
    uint32_t raw_ok = 0;
    auto load_quads = [&](int chunk) {
        qok = 0;
#pragma unroll
        for (int m = 0; m < SM; ++m) {
            const int ci_l = (lane + 64 * m) / (4 * KV);
            const int ci = chunk * CIC + (ci_l < CIC ? ci_l : 0);
            qok |= (ci < g.C_in ? 1u : 0u) << m;
            qraw[m] = win_load<W1>(p.x, geo, (uint32_t)min(ci, g.C_in - 1) * plane_bytes);
        }
    };
    // !QUAD: lane extracts pixel (lane % 16) for input channels lane / 16 + 4 m
    auto load_windows = [&](int chunk) {
        raw_ok = 0;
#pragma unroll
        for (int m = 0; m < WM; ++m) {
            const int ci = chunk * CIC + (lane >> 4) + 4 * m;
            raw_ok |= (ci < g.C_in ? 1u : 0u) << m;
            raw[m] = win_load<W1>(p.x, geo, (uint32_t)min(ci, g.C_in - 1) * plane_bytes);
        }
    };
    auto store_windows = [&]() {
#pragma unroll
        for (int m = 0; m < WM; ++m) {
            uint32_t row[3];
            win_rows(raw[m], geo, row);
            const uint32_t w = ((raw_ok >> m) & 1u) ? win_pick(row, 0) : 512u;
            wbuf[((lane >> 4) + 4 * m) * 16 + (lane & 15)] = (uint16_t)w;
        }
    };
    auto stage1 = [&]() {
#pragma unroll
        for (int m = 0; m < SM; ++m) {
            const int it = lane + 64 * m;
            if (ITEMS % 64 != 0 && it >= ITEMS) break;
            const int wd = it & 3;
            const int kv = (it >> 2) % KV;
            const int ci_l = it / (4 * KV);
            uint32_t w0, w1, w2, w3;
            if constexpr (QUAD) {
                uint32_t row[3];
                win_rows(qraw[m], geo, row);
                const bool ok = (qok >> m) & 1u;
                w0 = ok ? win_pick(row, 0) : 512u;
                w1 = ok ? win_pick(row, sstep) : 512u;
                w2 = ok ? win_pick(row, 2 * sstep) : 512u;
                w3 = ok ? win_pick(row, 3 * sstep) : 512u;
            } else {
                const uint2 w4 = *(const uint2 *)(wbuf + ci_l * 16 + 4 * wd);
                w0 = w4.x & 0xffffu;
                w1 = w4.x >> 16;
                w2 = w4.y & 0xffffu;
                w3 = w4.y >> 16;
            }
            const uint4 v0 = *(const uint4 *)(lut + w0 * LROW + kv * 16);
            const uint4 v1 = *(const uint4 *)(lut + w1 * LROW + kv * 16);
            const uint4 v2 = *(const uint4 *)(lut + w2 * LROW + kv * 16);
            const uint4 v3 = *(const uint4 *)(lut + w3 * LROW + kv * 16);
            uint32_t o[16];
            transpose4x4(v0.x, v1.x, v2.x, v3.x, o + 0);
            transpose4x4(v0.y, v1.y, v2.y, v3.y, o + 4);
            transpose4x4(v0.z, v1.z, v2.z, v3.z, o + 8);
            transpose4x4(v0.w, v1.w, v2.w, v3.w, o + 12);
            uint32_t *Tw = (uint32_t *)(T + ci_l * TS + kv * 256) + wd;
#pragma unroll
            for (int i = 0; i < 16; ++i) Tw[i * 4] = o[i];
        }
    };
    // LDS accesses of one wave are executed in order; this only keeps the compiler from moving
    // them across the stage boundary and waits for outstanding LDS operations.
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0)
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    uint32_t acc[J][4], wide_e[J][4], wide_o[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = wide_e[j][w] = wide_o[j][w] = 0;

    const uint4 *obase = (const uint4 *)p.offs + lane_co;
    uint4 oa[J], ob[J];
    auto load_offs = [&](int chunk, uint4 dst[J]) {
#pragma unroll
        for (int j = 0; j < J; ++j) dst[j] = obase[(int64_t)chunk * p.COP + j];
    };

    load_offs(0, oa);
    if constexpr (QUAD) {
        load_quads(0);
    } else {
        load_windows(0);
    }

    int since_widen = 0;
    auto iteration = [&](int c, const uint4 ocur[J], uint4 onext[J]) {
        const bool more = c + 1 < p.nchunks;
        load_offs(more ? c + 1 : c, onext);
        if constexpr (!QUAD) {
            store_windows();
            load_windows(c + 1);
            wave_sync();
        }
        stage1();
        if constexpr (QUAD) load_quads(c + 1);
        wave_sync();

        if (since_widen == WCH) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
                    wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
                    acc[j][w] = 0;
                }
            since_widen = 0;
        }
        ++since_widen;
        const uint32_t lb = (uint32_t)(T - smem);
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const uint32_t ow[4] = {ocur[j].x, ocur[j].y, ocur[j].z, ocur[j].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 va = *(const uint4 *)(smem + add_lo16(ow[q], lb) + (2 * q) * TS);
                const uint4 vb = *(const uint4 *)(smem + add_hi16(ow[q], lb) + (2 * q + 1) * TS);
                acc[j][0] = acc[j][0] + va.x + vb.x;
                acc[j][1] = acc[j][1] + va.y + vb.y;
                acc[j][2] = acc[j][2] + va.z + vb.z;
                acc[j][3] = acc[j][3] + va.w + vb.w;
            }
            asm volatile("" : "+v"(acc[j][0]), "+v"(acc[j][1]), "+v"(acc[j][2]), "+v"(acc[j][3]) : : "memory");
        }
        wave_sync();                              // gathers done before the next chunk overwrites T
    };
    for (int c = 0; c < p.nchunks; c += 2) {
        iteration(c, oa, ob);
        if (c + 1 < p.nchunks) iteration(c + 1, ob, oa);
    }

    // ---- epilogue ---------------------------------------------------------------------------------------
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
            wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
        }
    float a[J];
#pragma unroll
    for (int j = 0; j < J; ++j) a[j] = lane_co + j < g.C_out ? p.alpha[lane_co + j] : 0.0f;
    int n = t_n, r = t_r, ho = t_ho, wo = t_wo;         // wave-uniform
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float out[J][4];
        int rr[4], nn[4];
        bool ok[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            ok[b] = p_tile + 4 * w + b < g.P;
            rr[b] = r;
            nn[b] = n;
            const int type = border_type(ho, wo, g.H, g.W, g.stride);
            const int base = border_valid_taps(type) * g.C_in;
            if (type == 0) {                            // interior pixel: nothing to correct
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                    const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                    out[j][b] = (float)(2 * M - base) * a[j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                    const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                    const int co = lane_co + j;
                    const int cr = co < g.C_out ? p.corr[co * 16 + type] : 0;
                    out[j][b] = (float)(2 * (M - cr) - base) * a[j];
                }
            }
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) ho = 0;
            }
            if (++r == g.HoWo) {
                r = 0;
                ++n;
            }
        }
        if (p.vec4 && ok[3]) {
            float *dst = p.y + ((int64_t)nn[0] * g.C_out + lane_co) * g.HoWo + rr[0];
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (lane_co + j < g.C_out)
                    *(float4 *)(dst + (int64_t)j * g.HoWo) = make_float4(out[j][0], out[j][1], out[j][2], out[j][3]);
        } else {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (ok[b] && lane_co + j < g.C_out)
                        p.y[((int64_t)nn[b] * g.C_out + lane_co + j) * g.HoWo + rr[b]] = out[j][b];
        }
    }
    }   // tile loop
}

// ---- direct kernel (any K; used for K > 64) ------------------------------------------------------------
// Same tile / gather structure with G = 4, without the pipelining: stage 1 is XOR + popcount.

template <int J, int NW>
__global__ __launch_bounds__(NW * 64)
void subbit_direct_kernel(const SbParams p, int CIC)
{
    constexpr int NT = NW * 64;
    constexpr int G = 4, TP = 64, CL = 16;
    constexpr int COW = CL * J;
    const Geom &g = p.g;
    const int K = g.K;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *T = smem;                                              // [CIC][K][TP]
    uint16_t *wins = (uint16_t *)(smem + (size_t)CIC * K * TP);           // [CIC][TP]
    uint32_t *lcodes = (uint32_t *)(wins + CIC * TP);                     // [K]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t p_tile = (int64_t)blockIdx.x * TP;
    const int gq = lane % G, cl = lane / G;
    const int lane_co = blockIdx.y * (COW * NW) + wave * COW + cl * J;

    for (int i = tid; i < K; i += NT) lcodes[i] = p.codes[i];
    const PixGeom geo = pix_geom(p_tile + (tid & 63), g);

    uint32_t acc[J][4], wide_e[J][4], wide_o[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[j][w] = wide_e[j][w] = wide_o[j][w] = 0;
    int since_widen = 0;
    __syncthreads();

    // offsets are laid out for chunks of 8: [chunk8][COP][8]
    for (int c0 = 0; c0 < g.C_in; c0 += CIC) {
        const int nci = min(CIC, g.C_in - c0);
        for (int ci_l = tid >> 6; ci_l < nci; ci_l += NW)
            wins[ci_l * TP + (tid & 63)] = (uint16_t)window9(p.x, geo, c0 + ci_l, g);
        __syncthreads();
        const int items = nci * K * (TP / 4);
        for (int i = tid; i < items; i += NT) {
            const int wd = i & 15;
            const int k = (i >> 4) % K;
            const int ci_l = (i >> 4) / K;
            const uint2 w4 = *(const uint2 *)(wins + ci_l * TP + 4 * wd);
            const uint32_t code = lcodes[k];
            const uint32_t m0 = 9u - __popc((w4.x & 0xffffu) ^ code);
            const uint32_t m1 = 9u - __popc((w4.x >> 16) ^ code);
            const uint32_t m2 = 9u - __popc((w4.y & 0xffffu) ^ code);
            const uint32_t m3 = 9u - __popc((w4.y >> 16) ^ code);
            ((uint32_t *)T)[i] = m0 | (m1 << 8) | (m2 << 16) | (m3 << 24);
        }
        __syncthreads();
        if (since_widen + nci > SB_WIDEN) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
                    wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
                    acc[j][w] = 0;
                }
            since_widen = 0;
        }
        since_widen += nci;
        const unsigned char *Tl = T + gq * 16;
        for (int ci_l = 0; ci_l < nci; ++ci_l) {
            const int ci = c0 + ci_l;
            const uint16_t *op = p.offs + ((int64_t)(ci >> 3) * p.COP + lane_co) * 8 + (ci & 7);
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint4 v = *(const uint4 *)(Tl + op[j * 8]);
                acc[j][0] += v.x;
                acc[j][1] += v.y;
                acc[j][2] += v.z;
                acc[j][3] += v.w;
            }
            Tl += (size_t)K * TP;
        }
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wide_e[j][w] += acc[j][w] & 0x00ff00ffu;
            wide_o[j][w] += (acc[j][w] >> 8) & 0x00ff00ffu;
        }
    const int64_t pl = p_tile + gq * 16;
    if (pl >= g.P) return;
    int n = (int)(pl / g.HoWo);
    int r = (int)(pl - (int64_t)n * g.HoWo);
    int ho = r / g.Wo, wo = r - ho * g.Wo;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const bool ok = pl + 4 * w + b < g.P;
            const int type = border_type(ho, wo, g.H, g.W, g.stride);
            const int base = border_valid_taps(type) * g.C_in;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int co = lane_co + j;
                if (ok && co < g.C_out) {
                    const uint32_t pair = (b & 1) ? wide_o[j][w] : wide_e[j][w];
                    const int M = (int)((pair >> (16 * (b >> 1))) & 0xffffu);
                    const int S = 2 * (M - p.corr[co * 16 + type]) - base;
                    p.y[((int64_t)n * g.C_out + co) * g.HoWo + r] = (float)S * p.alpha[co];
                }
            }
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) ho = 0;
            }
            if (++r == g.HoWo) {
                r = 0;
                ++n;
            }
        }
}

// ---- configuration ------------------------------------------------------------------------------------

struct SbCfg {
    int G, J, NW;
    int cob() const { return (64 / G) * J * NW; }
};

// Instantiated (G, J, NW) combinations of the table-lookup kernel (see SNN_LUT below).
const SbCfg kCfgs[] = {
    {4, 1, 1}, {4, 1, 2}, {4, 1, 4}, {4, 1, 8}, {4, 2, 8}, {4, 4, 8},   // 16 .. 512 channels, 64 pixels
    {2, 1, 4}, {2, 1, 8}, {2, 2, 8},                                    // 128, 256, 512 channels, 32 pixels
    {1, 1, 1}, {1, 1, 2}, {1, 1, 4}, {1, 1, 8},                         //  64, 128, 256, 512 channels, 16 pixels
};

int round16(int K) { return (K + 15) & ~15; }

size_t lut_lds_bytes(const SbCfg &c, int K, int CIC)
{
    const int KP = round16(K), TP = 16 * c.G;
    return (size_t)513 * (KP + 16) + (size_t)2 * CIC * (KP * TP + SB_TPAD) + (size_t)2 * CIC * TP * sizeof(uint16_t);
}

// Pick the tile of the workgroup kernel.  The workgroup covers all output channels when it can
// (stage 1 is then done once per pixel); the tile is the widest one that still leaves enough
// workgroups to spread over 256 CUs (measured: 64-pixel tiles win from ~190 tiles up, 16-pixel
// tiles below ~100).
SbCfg pick_cfg(const Geom &g, bool lut)
{
    if (!lut) {
        static const SbCfg d[] = {{4, 1, 1}, {4, 1, 2}, {4, 1, 4}, {4, 2, 4}, {4, 4, 4}};
        for (const SbCfg &c : d)
            if (g.C_out <= c.cob()) return c;
        return d[4];
    }
    if (const char *e = getenv("SNN_SUBBIT_TILE")) {      // tuning override: "G,J,NW"
        int G = 0, J = 0, NW = 0;
        if (sscanf(e, "%d,%d,%d", &G, &J, &NW) == 3)
            for (const SbCfg &c : kCfgs)
                if (c.G == G && c.J == J && c.NW == NW) return c;
    }
    int G = 4;
    if ((g.P + 63) / 64 < 192) G = (g.P + 31) / 32 >= 192 ? 2 : 1;
    if (G == 2 && g.C_out <= 64) G = 4;                   // no narrow configuration for few channels
    if (G == 1 && g.C_out <= 32) G = 4;
    const SbCfg *last = nullptr;
    for (const SbCfg &c : kCfgs) {
        if (c.G != G) continue;
        last = &c;
        if (g.C_out <= c.cob()) return c;
    }
    return *last;                                         // several channel blocks of the largest one
}

struct SbPlan {
    bool lut;
    bool wave;        // wave-private variant of the lookup kernel (many pixels)
    int wJ;           // its channel sets per lane (64 * wJ channels per workgroup)
    SbCfg cfg;
    int CIC;          // input channels per chunk
    int COP;          // C_out padded to whole channel blocks
    int nchunks;      // chunks of the offsets table (of CIC channels for the lut kernel, 8 otherwise)
    size_t lds;
    // workspace carve-up
    size_t off_codes, off_offs, off_corr, off_lut, bytes;
};

size_t wave_lds_bytes(int K)
{
    const int KP = round16(K);
    return (size_t)513 * (KP + 16) + (size_t)WV_NW * (WV_CIC * (KP * 16 + 16) + WV_CIC * 16 * sizeof(uint16_t));
}

SbPlan make_plan(const Geom &g)
{
    SbPlan pl;
    pl.lut = g.K <= SB_LUT_MAXK;
    pl.wave = false;
    pl.wJ = 0;
    pl.cfg = pick_cfg(g, pl.lut);
    int row_co = 0;       // output channels per workgroup (channel padding unit)
    if (pl.lut) {
        // Wave-private tiles when there are enough 16-pixel tiles to give every SIMD several waves.
        int wJ = 1;
        while (wJ < 8 && 64 * wJ < g.C_out) wJ *= 2;
        const int64_t wtiles = (g.P + 15) / 16 * ((g.C_out + 64 * wJ - 1) / (64 * wJ));
        const char *e = getenv("SNN_SUBBIT_WAVE");          // tuning override: 0 / 1
        const bool want = e ? (e[0] == '1') : (wtiles >= 2048 && !getenv("SNN_SUBBIT_TILE"));
        if (want) {
            pl.wave = true;
            pl.wJ = wJ;
        }
    }
    if (pl.wave) {
        pl.CIC = WV_CIC;
        pl.lds = wave_lds_bytes(g.K);
        pl.nchunks = (g.C_in + pl.CIC - 1) / pl.CIC;
        row_co = 64 * pl.wJ;
    } else if (pl.lut) {
        pl.CIC = lut_lds_bytes(pl.cfg, g.K, 8) <= 64 * 1024 ? 8 : 4;
        pl.lds = lut_lds_bytes(pl.cfg, g.K, pl.CIC);
        pl.nchunks = (g.C_in + pl.CIC - 1) / pl.CIC;
        row_co = pl.cfg.cob();
    } else {
        int CIC = 8;
        while (CIC > 1 && (size_t)CIC * g.K * 64 > 32 * 1024) CIC >>= 1;
        pl.CIC = CIC;
        pl.lds = (size_t)CIC * g.K * 64 + (size_t)CIC * 64 * sizeof(uint16_t) + (size_t)g.K * sizeof(uint32_t);
        pl.nchunks = (g.C_in + 7) / 8;
        row_co = pl.cfg.cob();
    }
    pl.COP = (g.C_out + row_co - 1) / row_co * row_co;
    const int occ = pl.lut ? pl.CIC : 8;     // channels per offsets chunk
    size_t o = 0;
    pl.off_codes = o;
    o += align_up(512 * sizeof(uint32_t), 256);
    pl.off_offs = o;
    o += align_up((size_t)pl.nchunks * pl.COP * occ * sizeof(uint16_t), 256);
    pl.off_corr = o;
    o += align_up((size_t)pl.COP * 16 * sizeof(int32_t), 256);
    pl.off_lut = o;
    if (pl.lut) o += align_up((size_t)513 * (round16(g.K) + 16), 256);
    pl.bytes = o;
    return pl;
}

template <int J, int KP, int MODE>
int launch_wave_q(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    auto kern = subbit_wave_kernel<J, KP, MODE>;
    if (pl.lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds) != hipSuccess)
        return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, grid, dim3(WV_NW * 64), pl.lds, s, prm);
    return check_launch();
}

template <int J>
int launch_wave(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    const int KP = round16(prm.g.K);
    const int mode = ((prm.g.Wo & 3) == 0 ? 2 : 0) | (prm.g.WW == 1 ? 1 : 0);
#define SNN_WAVE_KP(KP_)                                                              \
    if (KP == KP_) switch (mode) {                                                    \
        case 0: return launch_wave_q<J, KP_, 0>(pl, prm, grid, s);                    \
        case 1: return launch_wave_q<J, KP_, 1>(pl, prm, grid, s);                    \
        case 2: return launch_wave_q<J, KP_, 2>(pl, prm, grid, s);                    \
        default: return launch_wave_q<J, KP_, 3>(pl, prm, grid, s);                   \
        }
    SNN_WAVE_KP(32)
#ifndef SNN_FAST_BUILD
    SNN_WAVE_KP(16)
    SNN_WAVE_KP(48)
    SNN_WAVE_KP(64)
#endif
#undef SNN_WAVE_KP
    return SNN_ERR_UNSUPPORTED;
}

template <int G, int J, int NW, int KP, int CIC, int MODE>
int launch_lut_w(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    auto kern = subbit_lut_kernel<G, J, NW, KP, CIC, MODE>;
    if (pl.lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds) != hipSuccess)
        return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), pl.lds, s, prm);
    return check_launch();
}

template <int G, int J, int NW, int KP, int CIC>
int launch_lut_one(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    const int mode = ((prm.g.Wo & 3) == 0 ? 2 : 0) | (prm.g.WW == 1 ? 1 : 0);
    switch (mode) {
    case 0: return launch_lut_w<G, J, NW, KP, CIC, 0>(pl, prm, grid, s);
    case 1: return launch_lut_w<G, J, NW, KP, CIC, 1>(pl, prm, grid, s);
    case 2: return launch_lut_w<G, J, NW, KP, CIC, 2>(pl, prm, grid, s);
    default: return launch_lut_w<G, J, NW, KP, CIC, 3>(pl, prm, grid, s);
    }
}

template <int G, int J, int NW>
int launch_lut(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    const int KP = round16(prm.g.K);
#define SNN_LUT_KP(KP_)                                                                        \
    if (KP == KP_)                                                                             \
        return pl.CIC == 8 ? launch_lut_one<G, J, NW, KP_, 8>(pl, prm, grid, s)                \
                           : launch_lut_one<G, J, NW, KP_, 4>(pl, prm, grid, s);
    SNN_LUT_KP(32)
#ifndef SNN_FAST_BUILD
    SNN_LUT_KP(16)
    SNN_LUT_KP(48)
    SNN_LUT_KP(64)
#endif
#undef SNN_LUT_KP
    return SNN_ERR_UNSUPPORTED;
}

template <int J, int NW>
int launch_direct(const SbPlan &pl, const SbParams &prm, dim3 grid, hipStream_t s)
{
    auto kern = subbit_direct_kernel<J, NW>;
    if (pl.lds > 64 * 1024 && hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                  (int)pl.lds) != hipSuccess)
        return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), pl.lds, s, prm, pl.CIC);
    return check_launch();
}

}  // namespace

int launch_subbit_f32(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                      const float *alpha, float *y, void *ws, hipStream_t s);
size_t subbit_f32_workspace_bytes(const Geom &g);

// The matrix-core kernel takes every layer it supports; SNN_SUBBIT_MFMA=0 (a tuning override)
// sends those layers to the LDS-gather kernels of this file instead.
static bool use_mfma(const Geom &g)
{
    const char *e = getenv("SNN_SUBBIT_MFMA");
    return subbit_mfma_supported(g) && !(e && e[0] == '0');
}

size_t subbit_workspace_bytes(const Geom &g, int act)
{
    if (act == SNN_ACT_F32) return subbit_f32_workspace_bytes(g);
    // sized for either kernel family, so that the override cannot outgrow a workspace
    const size_t a = make_plan(g).bytes;
    const size_t b = subbit_mfma_supported(g) ? subbit_mfma_workspace_bytes(g) : 0;
    return a > b ? a : b;
}

int launch_subbit(const Geom &g, int act, const void *x, const uint16_t *codebook, const uint16_t *idx,
                  const float *alpha, float *y, void *ws, hipStream_t s)
{
    if (act == SNN_ACT_F32) return launch_subbit_f32(g, x, codebook, idx, alpha, y, ws, s);
    if (use_mfma(g)) return launch_subbit_mfma(g, x, codebook, idx, alpha, y, ws, s);

    const SbPlan pl = make_plan(g);
    const SbCfg &c = pl.cfg;
    const int TP = pl.wave ? 16 : 16 * c.G;
    // wave-private variant: persistent workgroups, two per CU fit the LDS
    const int64_t wave_wgs = ((g.P + 15) / 16 + WV_NW - 1) / WV_NW;
    const int64_t tiles = pl.wave ? (wave_wgs < 512 ? wave_wgs : 512) : (g.P + TP - 1) / TP;
    const int cblocks = pl.wave ? pl.COP / (64 * pl.wJ) : pl.COP / c.cob();
    if (tiles > 0x7fffffffLL || cblocks > 65535 || pl.lds > 160 * 1024) return SNN_ERR_UNSUPPORTED;
    // the kernels address the packed input with 32-bit word offsets
    if ((int64_t)g.N * g.C_in * g.H * g.WW >= ((int64_t)1 << 31)) return SNN_ERR_UNSUPPORTED;

    SbParams prm;
    prm.x = (const uint32_t *)x;
    prm.codes = (const uint32_t *)((char *)ws + pl.off_codes);
    prm.offs = (const uint16_t *)((char *)ws + pl.off_offs);
    prm.corr = (const int32_t *)((char *)ws + pl.off_corr);
    prm.lut = (const uint4 *)((char *)ws + pl.off_lut);
    prm.alpha = alpha;
    prm.y = y;
    prm.g = g;
    prm.COP = pl.COP;
    prm.nchunks = pl.nchunks;
    prm.vec4 = ((g.HoWo & 3) == 0 && ((uintptr_t)y & 15) == 0) ? 1 : 0;

    const int occ = pl.lut ? pl.CIC : 8;
    const int64_t n_offs = (int64_t)pl.nchunks * pl.COP * occ;
    const int offs_blocks = (int)((n_offs + 255) / 256);
    const int corr_blocks = (pl.COP + 3) / 4;
    const int lut_blocks = pl.lut ? (513 * (round16(g.K) + 16) / 4 + 255) / 256 : 0;
    hipLaunchKernelGGL(subbit_prep_kernel, dim3((unsigned)(offs_blocks + corr_blocks + lut_blocks)), dim3(256), 0, s,
                       codebook, idx, g.C_in, g.C_out, pl.COP, g.K, occ, pl.nchunks, TP, offs_blocks, lut_blocks,
                       (uint32_t *)prm.codes, (uint16_t *)prm.offs, (int32_t *)prm.corr, (uint32_t *)prm.lut);

    const dim3 grid((unsigned)tiles, (unsigned)cblocks);
    if (pl.wave) {
        switch (pl.wJ) {
        case 1: return launch_wave<1>(pl, prm, grid, s);
        case 2: return launch_wave<2>(pl, prm, grid, s);
        case 4: return launch_wave<4>(pl, prm, grid, s);
        case 8: return launch_wave<8>(pl, prm, grid, s);
        default: return SNN_ERR_UNSUPPORTED;
        }
    }
    if (!pl.lut) {
#define SNN_DIRECT(J_, NW_) \
    if (c.J == J_ && c.NW == NW_) return launch_direct<J_, NW_>(pl, prm, grid, s);
        SNN_DIRECT(1, 1)
        SNN_DIRECT(1, 2)
        SNN_DIRECT(1, 4)
        SNN_DIRECT(2, 4)
        SNN_DIRECT(4, 4)
#undef SNN_DIRECT
        return SNN_ERR_UNSUPPORTED;
    }
#define SNN_LUT(G_, J_, NW_) \
    if (c.G == G_ && c.J == J_ && c.NW == NW_) return launch_lut<G_, J_, NW_>(pl, prm, grid, s);
    SNN_LUT(4, 1, 1)
    SNN_LUT(4, 1, 2)
    SNN_LUT(4, 1, 4)
    SNN_LUT(4, 1, 8)
    SNN_LUT(4, 2, 8)
    SNN_LUT(4, 4, 8)
    SNN_LUT(2, 1, 4)
    SNN_LUT(2, 1, 8)
    SNN_LUT(2, 2, 8)
    SNN_LUT(1, 1, 1)
    SNN_LUT(1, 1, 2)
    SNN_LUT(1, 1, 4)
    SNN_LUT(1, 1, 8)
#undef SNN_LUT
    return SNN_ERR_UNSUPPORTED;
}


}  // namespace snn
