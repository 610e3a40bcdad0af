// Sub-bit 3x3 convolution for K <= 64 on the matrix cores (Sec. 4.5 / Fig. 6).
//
// Stage 1 (responses of the K subset kernels, once per input channel and pixel) is a table
// lookup: the 9-bit window of +-1 activations selects a row of K match counts
// m_k = 9 - popcount(window ^ code_k) in [0, 9], taps outside the image forced to "no match" and
// corrected at the end.  Stage 2 (gather by index, sum over c_in) is written as a product with a
// one-hot matrix, contracted over (c_in, k):
//     M[co][pixel] = sum_ci sum_k  onehot(idx[co][ci])[k] * m_k(window[ci][pixel])
// One v_mfma_f32_32x32x64_f8f6f4 covers 32 output channels x 32 pixels and 64 contraction
// slots, of which lanes 0-31 supply the first 32 and lanes 32-63 the rest.  For K <= 32 the slots
// are (channel parity, subset member k): TWO input channels per instruction, the even one in the
// low lanes.  For 32 < K <= 64 they are the members k of ONE input channel.  For K <= 16 a lane
// half can hold two channels of 16 slots each, FOUR channels per instruction (used on long layers).
//   A operand (FP4 e2m1): the one-hot row of an output channel, 32 nibbles, made from a
//     pre-computed byte selector with four v_perm_b32;
//   B operand (FP6 e2m3): the table row itself, stored as m_k - 4 in [-4, 5] (exact in e2m3), read
//     from LDS as it is: the responses never need transposing or a trip through LDS;
//   accumulation in fp32 is exact (integers far below 2^24).
// S = 2 * (M' + 4 C_in - corr[co][border type]) - C_in * valid_taps with M' the accumulated sum,
// y = float(S) * alpha[co].
//
// A wave owns PB blocks of 32 pixels x CB blocks of 32 output channels and a range of input
// channel pairs; the KS waves that split the channels of one tile sit in one workgroup and add
// their partial sums through LDS.
#include "front_ops.h"
#include "subbit_mfma_plan.h"

#include <type_traits>

namespace snn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const u32x4 lds_cu32x4;
typedef __attribute__((address_space(3))) const u32x2 lds_cu32x2;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) const uint32_t lds_cu32;
typedef __attribute__((address_space(3))) uint32_t lds_u32;

constexpr uint32_t MF_SEL_NONE = 0x0c0c0c0cu;  // v_perm_b32 selector bytes that produce 0x00

struct MfParams {
    const uint32_t *x;        // packed rows [N][C_in][H][WW]
    const uint32_t *lut;      // [512][6 or 12] words: row = window, 32 (64) FP6 values m_k - 4 packed little-endian
    const uint32_t *sel;      // [steps][2][COP] selector words for the one-hot operand
    const uint2 *fin;         // [COP][16] per (output channel, border type): {2 corr + C_in (valid_taps - 8), alpha bits}
    float *y;
    // binarised output (sign epilogue) instead of y when sign_out != nullptr:
    // bit = ((float)S * alpha[co] + beta[co] >= 0), packed rows [N][C_out][H_out][ceil(W_out / 32)];
    // `fin` then holds thresholds (fin_entry)
    uint32_t *sign_out;
    int n_pxblocks;           // blocks of up to 32 pixels (see pixel_of)
    // 1x1 layers (WM == 3): x is packed channels [N][H][W][cw_bytes / 4]; g.C_in counts groups of 8 input channels
    uint32_t x_bytes, cw_bytes;
    Geom g;
    int COP;                  // C_out padded to whole wave tiles
    int KS;                   // waves that split the channel pairs of one tile: 1, 2 or 4
    int npairs;               // steps: (C_in + 1) / 2 of two input channels (K <= 32), C_in of one, or (C_in + 3) / 4 of four (QUAD)
    int pairs_per_split;
    int n_cotiles;
    long long n_tiles;        // pixel tiles * channel tiles
};

// FP6 e2m3 code of an integer in [-7, 7]
__host__ __device__ inline uint32_t fp6_of_int(int v)
{
    const uint32_t s = v < 0 ? 32u : 0u;
    const int a = v < 0 ? -v : v;
    // 0; 1 = 1.000 x 2^0; 2, 3 = 1.m x 2^1; 4 .. 7 = 1.m x 2^2  (bias 1, three mantissa bits)
    const uint32_t mag = a == 0 ? 0u : a == 1 ? 8u : a < 4 ? 16u + 4u * (uint32_t)(a - 2) : 24u + 2u * (uint32_t)(a - 4);
    return s | mag;
}

// ---- preparation: selector tables, finishing table, lookup table -----------------------------------
// Step c of the convolution handles channels (2c, 2c+1); for odd C_in the last step handles
// (C_in-2, C_in-1) and its first half is switched off.
//   sel[c][h][co]: k = idx[co][channel h of step c]; nibble k of the 32-nibble one-hot row is byte
//     k / 2 (word k / 8), low or high nibble.  Byte p of the selector is
//     (p == (k / 2) % 4) ? 2 (k / 8) + k % 2 : 0x0c, so that v_perm_b32 with the 8-byte constant
//     {0x02 at byte 2 j, 0x20 at byte 2 j + 1} yields word j of the row (FP4 1.0 = 0b0010).
//   fin[co][type] = {2 corr + C_in * (valid_taps(type) - 8), alpha[co]} with corr = sum over c_in of the
//     zero bits of the selected code at the taps that border type `type` puts outside the image
//   lut[window] = 32 FP6 codes of m_k - 4 (0 for k >= K)
// one thread per 32-bit word of the table; a row is 6 words of 32 FP6 codes per lane half
// `taps` = 9: 512 rows indexed by the 3x3 window; `taps` = 8 (1x1 layers): 256 rows indexed by the signs
// of 8 consecutive input channels, member element j at code bit 7 - j, channel 8 g + j at window bit j.
__device__ inline void prep_lut_block(const uint16_t *__restrict__ codebook, int K, int pair, int block, uint32_t *__restrict__ lut,
                                      int taps = 9)
{
    const int wpr = pair ? 6 : 12;
    const int i = block * 256 + (int)threadIdx.x;
    if (i < (taps == 9 ? 512 : 256) * wpr) {
        const int win = i / wpr, wh = i - win * wpr;
        const int half = wh / 6, w = wh - 6 * half;
        uint32_t word = 0;
        for (int kl = (32 * w) / 6; kl <= (32 * w + 31) / 6; ++kl) {
            const int k = 32 * half + kl;
            if (k >= K) break;
            const int m = taps == 9 ? 9 - __popc((uint32_t)win ^ code_to_window_order(codebook[k] & 511u))
                                    : 8 - __popc(((uint32_t)win ^ (__brev((uint32_t)codebook[k] & 255u) >> 24)) & 255u);
            const int at = 6 * kl - 32 * w;                // position of the code's bit 0 in this word
            const uint32_t code = fp6_of_int(m - 4);
            word |= at >= 0 ? code << at : code >> -at;
        }
        lut[i] = word;
        // the same table a second time for the kernel of subbit_stack.hip, behind the first image (whose region is
        // sized for 48-byte rows and holds 24-byte ones): the first four words of all rows, then the last two
        if (pair && taps == 9) lut[MF_LUT_SPLIT_WORDS + (w < 4 ? 4 * win + w : 2048 + 2 * win + (w - 4))] = word;
    }
}

// One entry of the finishing table, for output channel co and border type `type`:
//   corr_term = 2 corr + C_in (valid_taps(type) - 8), so that S = 2 acc - corr_term for the accumulator acc.
// fp32 output (beta == nullptr): {corr_term, alpha}; the epilogue computes y = float(S) * alpha.
// Sign epilogue: the bit (fl(fl(S * alpha) + beta) >= 0) is monotone in the integer S, so it equals
// S >= T (alpha > 0) or S <= T (alpha < 0) for a threshold T found here by bisection over all sums
// the layer can produce, with the very fp32 expression that defines the bit; folded with corr_term
// the entry is {mult, thr} (two floats) and the epilogue's test is acc * mult >= thr, exact
// because acc, mult and thr are small integers.  alpha = 0 or NaN: the bit does not depend on S (mult = 0).
__device__ inline uint2 fin_entry(int corr_term, float a, const float *beta, int co, bool real, int C_in)
{
    if (!beta) return make_uint2((uint32_t)corr_term, __float_as_uint(a));
    const float b = real ? beta[co] : 0.0f;
    const int smax = 9 * C_in;
    auto pred = [&](int S) { return mul_then_add((float)S, a, b) >= 0.0f; };
    float mult, thr;
    if (a > 0.0f || a < 0.0f) {
        // first S in [-smax, smax + 1] from which on the bit is 1 (a > 0) / 0 (a < 0)
        int lo = -smax, hi = smax + 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (pred(mid) == (a > 0.0f)) hi = mid;
            else lo = mid + 1;
        }
        if (a > 0.0f) {
            const int t = lo + corr_term;                       // 2 acc >= T + corr_term
            mult = 1.0f;
            thr = (float)((t + 1) >> 1);                        // ceil(t / 2)
        } else {
            const int t = (lo - 1) + corr_term;                 // 2 acc <= T + corr_term, T = lo - 1 the last S with bit 1
            mult = -1.0f;
            thr = -(float)(t >> 1);                             // -floor(t / 2)
        }
    } else {
        mult = 0.0f;
        thr = pred(0) ? -1.0f : 1.0f;
    }
    return make_uint2(__float_as_uint(mult), __float_as_uint(thr));
}

// Index i of an index tensor: plain uint16 (tau = 0), or tau bits at bit i * tau of a little-endian bit
// stream of 32-bit words (the storage format of Sec. 4.4 / Fig. 5: tau bits per kernel, tau / 9 per weight).
__device__ inline uint32_t index_at(const void *__restrict__ idx, int64_t i, int tau)
{
    if (tau == 0) return ((const uint16_t *)idx)[i];
    const uint32_t *w = (const uint32_t *)idx;
    const int64_t bit = i * tau;
    const int64_t word = bit >> 5;
    const int sh = (int)(bit & 31);
    uint32_t v = w[word] >> sh;
    if (sh + tau > 32) v |= w[word + 1] << (32 - sh);
    return v & ((1u << tau) - 1u);
}

// selector word of subset member k (see below)
__device__ inline uint32_t sel_word(uint32_t k)
{
    const uint32_t code = 2u * ((k >> 3) & 3u) + (k & 1u);       // k % 32 inside its lane half
    const int sh = 8 * ((k >> 1) & 3u);
    return (MF_SEL_NONE & ~(0xffu << sh)) | (code << sh);
}

// Stores the selector of (output channel co at position pos of a selector row, input channel ci)
// where the convolution's step / lane half expects it; k < 0: no member (padding channel).
__device__ inline void store_sel(uint32_t *__restrict__ sel, int COP, int C_in, int pair, int pos, int ci, int k)
{
    if (pair == 2) {
        // four channels per step (K <= 16): channel ci is slot-half (ci % 2) of lane half (ci / 2) % 2 of step
        // ci / 4; the second channel of a lane half owns slots 16 .. 31.  Channels from C_in up to the next
        // multiple of four get "no member" (the caller passes them with k < 0).
        const int c = ci >> 2, h = (ci >> 1) & 1, j = ci & 1;
        sel[(((int64_t)c * 2 + h) * 2 + j) * COP + pos] = k >= 0 ? sel_word((uint32_t)k + 16u * (uint32_t)j) : MF_SEL_NONE;
        return;
    }
    const uint32_t s = k >= 0 ? sel_word((uint32_t)k) : MF_SEL_NONE;
    if (!pair) {
        // one channel per step; the member's half (k / 32) gets the selector, the other one nothing
        const int hk = k >= 32 ? 1 : 0;
        sel[((int64_t)ci * 2 + hk) * COP + pos] = s;
        sel[((int64_t)ci * 2 + (hk ^ 1)) * COP + pos] = MF_SEL_NONE;
        return;
    }
    // channel ci is half (ci % 2) of step ci / 2, except the last channel of an odd C_in
    int c = ci >> 1, h = ci & 1;
    if ((C_in & 1) && ci == C_in - 1) {
        c = (C_in + 1) / 2 - 1;
        h = 1;
        sel[((int64_t)c * 2 + 0) * COP + pos] = MF_SEL_NONE;
    }
    sel[((int64_t)c * 2 + h) * COP + pos] = s;
}

// Tables for the launch that walks a stack of layers (fp32 output): the finishing table again, laid out
// so that a lane reads the entries of four consecutive output channels with one access:
// negcorr[type][co] = -(2 corr + C_in (valid_taps(type) - 8)) as int16 (|.| <= 10 C_in, C_in <= 3000),
// alphap[co] = alpha (0 for padding channels); and the scheduling words, zeroed.
struct StackTables {
    int16_t *negcorr;
    float *alphap;
    uint32_t *sched;
    int COP;
};
__device__ inline void store_stack_entry(const StackTables &st, int co, int type, int corr_term, float a)
{
    st.negcorr[type * st.COP + co] = (int16_t)(-corr_term);
    if (type == 0) st.alphap[co] = a;
}

__global__ __launch_bounds__(256)
void subbit_mfma_prep_kernel(const uint16_t *__restrict__ codebook, const void *__restrict__ idx, int tau, int C_in,
                             int C_out, int COP, int CB, int K, int pair, int sel_blocks, int lut_blocks,
                             const float *__restrict__ alpha, uint32_t *__restrict__ sel, uint2 *__restrict__ fin,
                             uint32_t *__restrict__ lut, const float *__restrict__ beta, int taps, StackTables st)
{
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    if (b == (int)gridDim.x - 1)
        for (int i = tid; i < MF_SCHED_WORDS; i += 256) st.sched[i] = 0u;
    if (b < sel_blocks) {
        // tile of 32 output channels x 32 input channels: read along c_in, write along c_out
        __shared__ uint16_t tile[32][33];
        const int cot = COP / 32;
        const int co0 = (b % cot) * 32, ci0 = (b / cot) * 32;
        for (int e = tid; e < 1024; e += 256) {
            const int co = co0 + e / 32, ci = ci0 + e % 32;
            tile[e / 32][e % 32] = (co < C_out && ci < C_in) ? (uint16_t)min((int)index_at(idx, (int64_t)co * C_in + ci, tau), K - 1) : 0xffffu;
        }
        __syncthreads();
        for (int e = tid; e < 1024; e += 256) {
            const int co_l = e % 32, ci_l = e / 32;
            const int ci = ci0 + ci_l;
            if (ci >= (pair == 2 ? (C_in + 3) / 4 * 4 : C_in)) continue;
            const uint32_t k = tile[co_l][ci_l];
            // position inside a row of COP selectors: [wave tile][channel in block][block]
            const int co = co0 + co_l, tilew = 32 * CB;
            const int pos = (co / tilew) * tilew + (co % 32) * CB + (co % tilew) / 32;
            store_sel(sel, COP, C_in, pair, pos, ci, k == 0xffffu ? -1 : (int)k);
        }
        return;
    }
    if (b >= (int)gridDim.x - lut_blocks) {
        prep_lut_block(codebook, K, pair, b - ((int)gridDim.x - lut_blocks), lut, taps);
        return;
    }
    if (taps == 8) {
        // 1x1 layers have no border: S = 2 acc, nothing to correct
        const int co = (b - sel_blocks) * 4 + (tid >> 6);
        if (co < COP && (tid & 63) < 16) {
            fin[co * 16 + (tid & 63)] = make_uint2(0u, __float_as_uint(co < C_out ? alpha[co] : 0.0f));
            store_stack_entry(st, co, tid & 63, 0, co < C_out ? alpha[co] : 0.0f);
        }
        return;
    }
    // one wave per output channel; the zero-bit patterns of the K codes go through LDS so that the
    // loop over the input channels has one memory access per channel, not two dependent ones
    __shared__ uint32_t zbits[512];
    for (int k = tid; k < K; k += 256) zbits[k] = ~code_to_window_order(codebook[k] & 511u) & 511u;
    __syncthreads();
    const int co = (b - sel_blocks) * 4 + (tid >> 6);
    const int lane = tid & 63;
    if (co >= COP) return;
    int zeros[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) zeros[t] = 0;
    if (co < C_out)
        for (int c0 = 0; c0 < C_in; c0 += 256) {
            int kk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ci = c0 + 64 * u + lane;
                kk[u] = ci < C_in ? min((int)index_at(idx, (int64_t)co * C_in + ci, tau), K - 1) : -1;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t z = kk[u] >= 0 ? zbits[kk[u]] : 0u;
#pragma unroll
                for (int t = 0; t < 9; ++t) zeros[t] += __popcll(__ballot((z >> t) & 1u));
            }
        }
    if (lane < 16) {
        const uint32_t inv = border_invalid_window(lane);
        int s = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((inv >> t) & 1u) s += zeros[t];
        const float a = co < C_out ? alpha[co] : 0.0f;
        fin[co * 16 + lane] = fin_entry(2 * s + (border_valid_taps(lane) - 8) * C_in, a, beta, co, co < C_out, C_in);
        if (!beta) store_stack_entry(st, co, lane, 2 * s + (border_valid_taps(lane) - 8) * C_in, a);
    }
}

// ---- fused front kernel of snn_subbit_forward -----------------------------------------------------------
// Everything the convolution needs, in ONE launch whose blocks play three roles (block index ranges
// in this order, the long dependent chains first):
//   [0, COP)            one block per output channel: projection of its C_in real-valued kernels
//                       (Eq. 2 / Eq. 5) -> idx_out, selector words, finishing table row
//   [COP, +lut_blocks)  the lookup table
//   the rest            sign + packing of the activations into packed rows (Alg. 1: sign(a)); none when the
//                       input is packed already
// The few channel blocks ride along with the bandwidth-bound packing blocks instead of costing two
// launches of their own.
// The weights-side work of one layer (what the channel and table roles need).
struct WeightParams {
    const float *w;           // [C_out][C_in][9]
    const uint16_t *codebook;
    const float *alpha;
    const float *beta;        // sign epilogue: the finishing table holds thresholds (see fin_entry); else nullptr
    uint16_t *idx_out;        // [C_out][C_in]
    uint32_t *sel;
    uint2 *fin;
    uint32_t *lut;
    int C_in, C_out, COP, CB, K, pair, lut_blocks;
    StackTables st;
};
constexpr int FRONT_LDS_WORDS = 64 * 12 + 64 + 4 * 9;   // coef[K][12] floats, zero-bit patterns, per-wave counts

// One block = one output channel `co` of a layer: projection of its C_in kernels, index out,
// selector words, finishing table row.  A thread projects two kernels at a time (input channels
// tid and tid + 256 of a group of 512); the kernels of the first group are requested before
// anything else, those of the next group before the current one is worked on, so that the block
// waits for memory once.
__device__ inline void weight_channel_block(const WeightParams &p, int co, uint32_t *lds)
{
    const int tid = threadIdx.x;
    const int K = p.K, C_in = p.C_in;
    const int lane = tid & 63, wave = tid >> 6;
    const bool real = co < p.C_out;               // channels past C_out pad the last wave tile: no member, no output
    auto load_kernels = [&](int c0, float (&d)[2][9]) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int ci = c0 + 256 * q + tid;
            const bool have = real && ci < C_in;
            const float *src = p.w + ((int64_t)co * C_in + ci) * 9;
#pragma unroll
            for (int t = 0; t < 9; ++t) d[q][t] = have ? src[t] : 0.0f;
        }
    };
    float wt[2][9];
    load_kernels(0, wt);
    const float a = real ? p.alpha[co] : 0.0f;     // needed last, requested first
    float *coef = (float *)lds;
    uint32_t *zbits = lds + 64 * 12;
    uint32_t *wsum = zbits + 64;
    project_fill_coef(coef, p.codebook, K, tid, 256);
    for (int k = tid; k < K; k += 256) zbits[k] = ~code_to_window_order(p.codebook[k] & 511u) & 511u;
    __syncthreads();
    const int tilew = 32 * p.CB;
    const int pos = (co / tilew) * tilew + (co % 32) * p.CB + (co % tilew) / 32;
    int zeros[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) zeros[t] = 0;
    for (int c0 = 0; c0 < C_in; c0 += 512) {
        float nx[2][9];
        if (c0 + 512 < C_in) load_kernels(c0 + 512, nx);
        // waves whose 64 input channels lie past C_in have nothing to project; with at most 256 channels
        // left in the group the second kernel of every thread is empty as well (all wave-uniform)
        int best[2] = {0, 0};
        const int wave_ci = c0 + (tid & ~63);
        if (real && wave_ci + 256 < C_in) {
            project_argmax<2>(wt, coef, K, best);
        } else if (real && wave_ci < C_in) {
            int b1[1];
            project_argmax<1>(*(const float (*)[1][9]) & wt[0], coef, K, b1);
            best[0] = b1[0];
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int ci = c0 + 256 * q + tid;
            if (ci < C_in) {
                if (real) p.idx_out[(int64_t)co * C_in + ci] = (uint16_t)best[q];
                store_sel(p.sel, p.COP, C_in, p.pair, pos, ci, real ? best[q] : -1);
            }
            const uint32_t z = (real && ci < C_in) ? zbits[best[q]] : 0u;
#pragma unroll
            for (int t = 0; t < 9; ++t) zeros[t] += __popcll(__ballot((z >> t) & 1u));
        }
        if (c0 + 512 < C_in) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int t = 0; t < 9; ++t) wt[q][t] = nx[q][t];
        }
    }
    if (p.pair == 2 && C_in + tid < (C_in + 3) / 4 * 4) store_sel(p.sel, p.COP, C_in, 2, pos, C_in + tid, -1);
    if (lane == 0) {
#pragma unroll
        for (int t = 0; t < 9; ++t) wsum[wave * 9 + t] = (uint32_t)zeros[t];
    }
    __syncthreads();
    if (tid < 16) {
        const uint32_t inv = border_invalid_window(tid);
        int sum = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t)
            if ((inv >> t) & 1u) sum += (int)(wsum[t] + wsum[9 + t] + wsum[18 + t] + wsum[27 + t]);
        p.fin[co * 16 + tid] = fin_entry(2 * sum + (border_valid_taps(tid) - 8) * C_in, a, p.beta, co, real, C_in);
        if (!p.beta) store_stack_entry(p.st, co, tid, 2 * sum + (border_valid_taps(tid) - 8) * C_in, a);
    }
    if (co == 0)
        for (int i = tid; i < MF_SCHED_WORDS; i += 256) p.st.sched[i] = 0u;
}

struct FrontParams {
    const float *x;           // activations [rows][W]
    uint32_t *xr;             // packed rows
    int64_t rows;
    int W, WW, rows_per_block, vec;
    int64_t pack_blocks;      // 0: the activations are packed already
    WeightParams wp;
};

__global__ __launch_bounds__(256)
void subbit_front_kernel(const FrontParams p)
{
    static_assert(PACK_THREADS == 256, "one block size for all roles");
    static_assert(PACK_LDS_WORDS <= FRONT_LDS_WORDS, "the packing role's bit stream fits");
    __shared__ __align__(16) uint32_t lds[FRONT_LDS_WORDS];
    const int b = blockIdx.x;
    if (b >= p.wp.COP + p.wp.lut_blocks) {
        pack_rows_block(p.x, p.xr, p.rows, p.W, p.WW, p.rows_per_block, p.vec, (int64_t)(b - p.wp.COP - p.wp.lut_blocks), lds);
        return;
    }
    if (b >= p.wp.COP) {
        prep_lut_block(p.wp.codebook, p.wp.K, p.wp.pair, b - p.wp.COP, p.wp.lut);
        return;
    }
    weight_channel_block(p.wp, b, lds);
}

// The weights-side work of up to PREP_MANY_MAX layers in ONE launch (projection, selector /
// finishing / lookup tables of every layer): the blocks of layer l are [first_block[l], first_block[l + 1]),
// COP channel blocks followed by the table blocks.
constexpr int PREP_MANY_MAX = 32;
struct PrepManyParams {
    int n_layers;
    int first_block[PREP_MANY_MAX + 1];
    WeightParams layer[PREP_MANY_MAX];
};

__global__ __launch_bounds__(256)
void subbit_prepare_many_kernel(const PrepManyParams p)
{
    __shared__ __align__(16) uint32_t lds[FRONT_LDS_WORDS];
    const int b = blockIdx.x;
    int l = 0;
    while (l + 1 < p.n_layers && b >= p.first_block[l + 1]) ++l;      // block-uniform
    const WeightParams &wp = p.layer[l];
    const int lb = b - p.first_block[l];
    if (lb >= wp.COP) {
        prep_lut_block(wp.codebook, wp.K, wp.pair, lb - wp.COP, wp.lut);
        return;
    }
    weight_channel_block(wp, lb, lds);
}

// Buffer accesses: a scalar resource descriptor and scalar offset carry the wave-uniform part of the
// address (tensor base, input channel / output channel), the lane supplies a 32-bit byte offset: no
// address arithmetic in the vector ALU.  Lane offsets past the end of the buffer read as zero
// and are not stored.
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ inline void buf_store(__amdgpu_buffer_rsrc_t r, float v, uint32_t lane_off, uint32_t uniform_off)
{
    // non-temporal: the output is written once and not read again by this kernel; marked so, it drains to
    // memory while the kernel runs instead of sitting in L2 until the write-back at the kernel's end
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)lane_off, (int)uniform_off, 2 /* nt */);
}
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef __attribute__((address_space(3))) const u32x3 lds_cu32x3;
__device__ inline uint32_t buf_load1(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)uniform_off, 0);
}
__device__ inline u32x2 buf_load2(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, (int)uniform_off, 0);
}
__device__ inline u32x3 buf_load3(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b96(r, (int)lane_off, (int)uniform_off, 0);
}
__device__ inline u32x4 buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)uniform_off, 0);
}

// ---- the convolution ------------------------------------------------------------------------------
// PB, CB: blocks of 32 pixels / 32 output channels per wave.  WM: words per packed row, 1 or 2
// (the three window rows of a lane are then one contiguous load), or 0 for wider rows.
// PAIR: two input channels per step (K <= 32), else one (K <= 64); QUAD (with PAIR): four (K <= 16).
// STG: the packed rows a tile touches are few (at most MF_STAGE_SLOTS pieces per channel, WM = 1
// or 2).  Then the lanes do not fetch their own three rows from memory, 31 of 32 of those reads
// being the same words: per step ONE load brings every piece the wave needs (lane s of a half:
// piece s of the run of rows that starts at the first pixel's top row), the wave passes it through
// a private piece of LDS, and every lane reads ONE 32-bit piece per row from there.  A row of one
// word is one piece; a row of two words is three overlapping pieces, bits [0,32), [16,48) and
// [32,64), so that every window of three columns lies inside one of them.  The memory pipeline,
// which otherwise bounds the layers with few output channels, sees one instruction instead of 3 PB.
// `block` is the workgroup's number inside the layer (the launch of one layer passes blockIdx.x, the
// launch that walks several layers the offset from the layer's first workgroup); `smem` the
// workgroup's dynamic LDS.
template <int PB, int CB, int WM, bool PAIR, bool STG, bool QUAD = false>
__device__ __forceinline__ void mf_tile_body(const MfParams &p, const unsigned block, unsigned char *const smem)
{
    static_assert(!STG || WM == 1 || WM == 2, "staging needs rows that are consecutive in memory");
    // QUAD: subsets of at most 16 members.  A lane half then holds TWO input channels per step (channels
    // 4 c + 2 h and 4 c + 2 h + 1): 16 table values each in its operand, and two one-hot selectors, the
    // second one in slots 16 .. 31.  Half as many steps, twice the window work per step.
    static_assert(!QUAD || (PAIR && !STG && WM != 3), "four channels per step: 3x3 layers, rows loaded directly");
    // WM == 3: a 1x1 layer.  The "window" of a pixel and step is the byte of the signs of 8 consecutive
    // input channels (packed-channels input), a "channel" of the steps is such a group of 8, the table
    // has 256 rows of match counts m_k - 4 out of 8, there is no border, and S = 2 acc.
    constexpr bool ONE = WM == 3;
    constexpr int NBLK = PB * CB;
    constexpr int MF_LROW = mf_lrow(PAIR);
    const Geom &g = p.g;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_l = lane & 31, h = lane >> 5;

    const int KS = p.KS;
    const int split = wave & (KS - 1);
    const int tile_in_wg = wave / KS;
    const long long tile = (long long)block * (MF_WAVES / KS) + tile_in_wg;
    const bool active = tile < p.n_tiles;                       // wave-uniform
    const long long tl = active ? tile : p.n_tiles - 1;
    const int co_tile = (int)(tl % p.n_cotiles);
    const int blk0 = (int)(tl / p.n_cotiles) * PB;              // first pixel block of the tile
    const int co0 = co_tile * (32 * CB);

    // Pixel blocks.  For the fp32 output, block B is pixels 32 B .. 32 B + 31 of the flattened
    // (n, ho, wo) order.  For the sign epilogue a block is made of whole output words instead, so
    // that the wave that owns a block owns the words it writes: whole rows while they fit 32 pixels
    // (W_out <= 32: floor(32 / W_out) rows per block), else one 32-pixel word of a row; the lanes
    // left over are idle (12.5 % for rows of 7, 14, 28 or 56 pixels).  Either way the pixels of a tile
    // lie within 32 PB consecutive pixels of the flattened order.  Idle lanes and blocks past the end
    // work on the first pixel of their (or the last) block and are not written.
    const int P32 = (int)g.P;
    const bool aligned = p.sign_out != nullptr;
    const int rows_pb = g.Wo <= 32 ? 32 / g.Wo : 1;             // aligned, short rows: rows per block
    const int bpi = (g.Ho + rows_pb - 1) / rows_pb;             //   blocks per image
    const int wpr = (g.Wo + 31) / 32;                           // aligned, long rows: blocks (words) per row
    auto pixel_of = [&](int pb, int lane_px, int &n, int &ho, int &wo) -> bool {
        int B = blk0 + pb;
        bool ok = B < p.n_pxblocks;
        if (!ok) B = p.n_pxblocks - 1;
        if (!aligned) {
            int pp = B * 32 + lane_px;
            if (pp >= P32) {
                ok = false;
                pp = P32 - 1;
            }
            n = pp / g.HoWo;
            const int r = pp - n * g.HoWo;
            ho = r / g.Wo;
            wo = r - ho * g.Wo;
        } else if (g.Wo <= 32) {
            n = B / bpi;
            const int rb = B - n * bpi;
            int rl = lane_px / g.Wo;
            wo = lane_px - rl * g.Wo;
            if (rl >= rows_pb || rb * rows_pb + rl >= g.Ho) {
                ok = false;
                rl = 0;
                wo = 0;
            }
            ho = rb * rows_pb + rl;
        } else {
            const int R = B / wpr, j = B - R * wpr;
            n = R / g.Ho;
            ho = R - n * g.Ho;
            wo = 32 * j + lane_px;
            if (wo >= g.Wo) {
                ok = false;
                wo = 32 * j;
            }
        }
        return ok;
    };

    // The lookup table image was built once by the preparation kernel.  Its words are requested
    // first of all, so that they travel while the lanes work out their geometry.
    constexpr int HALVES = PAIR ? 1 : 2;
    constexpr int LUT_WORDS = (WM == 3 ? 256 : 512) * 6 * HALVES / (MF_WAVES * 64);     // per thread
    uint32_t lutw[LUT_WORDS];
#pragma unroll
    for (int i = 0; i < LUT_WORDS; ++i) lutw[i] = p.lut[i * (MF_WAVES * 64) + tid];
    __builtin_amdgcn_sched_barrier(0);

    // ---- per-lane window geometry of the PB pixels (pixel n_l of every block) ----------------------
    // This lane looks at input channel (2 c + h) in step c (PAIR; else channel c).  It loads three consecutive packed rows
    // starting at row max(hc - 1, 0), words (jlo, jlo + 1), and cuts row dy of the window out of the
    // 64-bit string {hi, lo} at bit `sh`.  Two cases are folded into a final shift `lsh` of the
    // 9-bit window so that no load starts before the tensor:
    //   top image row   : the rows loaded are (hc, hc + 1, hc + 2), i.e. window rows 1, 2, 3 -> shift by 3;
    //   first image column: the bits cut out are columns (0, 1, 2) -> keep two (`m7` = 3), shift by 1.
    // Nothing else is clamped: words from outside the row, the image or the tensor (the latter read
    // as zero) only reach window bits whose taps lie outside the image, and `vm` masks those off.
    const uint32_t plane_bytes = (uint32_t)(g.H * g.WW) * 4u;
    uint32_t xoff[PB];                             // byte offset of the first word loaded, channel h of the pixel's image
    uint32_t sh[PB], m7[PB], lsh[PB], vm[PB];
    uint32_t yoff[PB];                             // byte offset of y[n][4 h][pixel], out of range for pixels past the end
    int ptype[PB];                                 // border type
    // Staging (STG): rows are numbered R = n * H + h over the whole batch; the wave stages words
    // [0, MF_STAGE_SLOTS) of the run of rows that starts at R_first, the first row the tile's
    // first pixel loads.  A pixel's three rows start (R - R_first) * WM + jlo words into the run.
    const uint32_t stage_wave = (uint32_t)(uintptr_t)smem + 512u * (uint32_t)MF_LROW + (uint32_t)wave * MF_STAGE_BYTES;
    constexpr int SW = WM == 2 ? 3 : 1;            // pieces per staged row
    int R_first = 0;
    uint32_t goff = 0xffffffffu;                   // byte offset of the word(s) this lane stages (channel h of the step)
    uint32_t gshift = 0;                           // two-word rows: the piece is bits [gshift, gshift + 32) of the two words loaded
    uint32_t loff[PB];                             // LDS address of the pixel's piece of its first row
    if constexpr (STG) {
        int n0, ho0, wo0;
        pixel_of(0, 0, n0, ho0, wo0);              // the tile's first pixel (wave-uniform)
        const int hc0 = ho0 * g.stride;
        R_first = n0 * g.H + (hc0 == 0 ? 0 : hc0 - 1);
        const int R = R_first + n_l / SW, piece = n_l % SW;
        const int n = R / g.H, hr = R - n * g.H;
        if (n < g.N && (PAIR || h == 0))
            goff = (uint32_t)(((n * g.C_in + (PAIR ? h : 0)) * g.H + hr) * g.WW + (piece == 2 ? 1 : 0)) * 4u;
        gshift = piece == 1 ? 16u : 0u;
    }
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        int n, ho, wo;
        const bool ok = pixel_of(pb, n_l, n, ho, wo);
        yoff[pb] = ok ? (uint32_t)((n * g.C_out + 4 * h) * g.HoWo + ho * g.Wo + wo) * 4u : 0xffffffffu;
        if constexpr (ONE) {
            ptype[pb] = 0;
            xoff[pb] = (uint32_t)((n * g.H + ho * g.stride) * g.W + wo * g.stride) * p.cw_bytes;
            sh[pb] = m7[pb] = lsh[pb] = vm[pb] = loff[pb] = 0;
            continue;
        }
        ptype[pb] = border_type(ho, wo, g.H, g.W, g.stride);
        vm[pb] = ~border_invalid_window(ptype[pb]) & 0x1ffu;
        const int hc = ho * g.stride, first = wo * g.stride - 1;
        const int col = first < 0 ? 0 : first;     // column of the first bit cut out
        const int jlo = WM == 1 ? 0 : col >> 5;
        const int piece = WM == 2 ? (col < 30 ? 0 : col < 46 ? 1 : 2) : 0;          // staged piece that holds columns col .. col + 2
        sh[pb] = STG ? (uint32_t)(col - 16 * piece) : (uint32_t)(col & 31);
        m7[pb] = first < 0 ? 3u : 7u;
        lsh[pb] = (first < 0 ? 1u : 0u) + (hc == 0 ? 3u : 0u);
        xoff[pb] = (uint32_t)(((n * g.C_in + (QUAD ? 2 * h : PAIR ? h : 0)) * g.H + (hc == 0 ? 0 : hc - 1)) * g.WW + jlo) * 4u;
        loff[pb] = stage_wave + (uint32_t)((PAIR ? h * MF_STAGE_SLOTS : 0) + (n * g.H + (hc == 0 ? 0 : hc - 1) - R_first) * SW + piece) * 4u;
    }
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(p.x, ONE ? p.x_bytes : (uint32_t)g.N * (uint32_t)g.C_in * plane_bytes);
    const uint32_t lut_base = (uint32_t)(uintptr_t)smem;

    constexpr bool ONE_WORD = WM == 1 || STG;      // a lane cuts its window row out of one 32-bit piece
    struct Raw {
        uint32_t lo[PB][3], hi[ONE_WORD || ONE ? 1 : PB][3];
        uint32_t lo2[QUAD ? PB : 1][3], hi2[QUAD && !ONE_WORD ? PB : 1][3];      // QUAD: the lane half's second channel
        uint32_t byte_shift;                       // 1x1: position of the lane's group inside the word loaded
    };
    // step c -> first channel of the pair (the last step of an odd C_in starts one channel early)
    const int last_first = g.C_in - 2;
    const uint32_t row_bytes = (uint32_t)g.WW * 4u;
    auto load_raw = [&](int c, Raw &r) {
        if constexpr (ONE) {
            // the word that holds the lane's group of 8 channels (4 groups per word)
            const uint32_t grp = (uint32_t)(PAIR ? min(2 * c, last_first) + h : c);
            const uint32_t word_off = (grp >> 2) << 2;
            r.byte_shift = (grp & 3u) << 3;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) r.lo[pb][0] = buf_load1(xres, xoff[pb] + word_off, 0u);
            return;
        }
        // QUAD: channels 4 c + 2 h + {0, 1}; those past C_in read the next image or, past the tensor, zeros:
        // their selectors say "no member"
        const uint32_t co = (uint32_t)(QUAD ? 4 * c : PAIR ? min(2 * c, last_first) : c) * plane_bytes;
        auto rows_of = [&](uint32_t cof, uint32_t (&lo)[3], uint32_t (&hi)[3], int pb) {
            if constexpr (WM == 1) {                 // rows are consecutive words
                const u32x3 v = buf_load3(xres, xoff[pb], cof);
                lo[0] = v.x;
                lo[1] = v.y;
                lo[2] = v.z;
            } else if constexpr (WM == 2) {          // rows are consecutive word pairs
                const u32x4 v = buf_load4(xres, xoff[pb], cof);
                const u32x2 w = buf_load2(xres, xoff[pb] + 16u, cof);
                lo[0] = v.x;
                hi[0] = v.y;
                lo[1] = v.z;
                hi[1] = v.w;
                lo[2] = w.x;
                hi[2] = w.y;
            } else {
#pragma unroll
                for (int dy = 0; dy < 3; ++dy) {
                    const u32x2 v = buf_load2(xres, xoff[pb] + (uint32_t)dy * row_bytes, cof);
                    lo[dy] = v.x;
                    hi[dy] = v.y;
                }
            }
        };
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            rows_of(co, r.lo[pb], r.hi[ONE_WORD ? 0 : pb], pb);
            if constexpr (QUAD) rows_of(co + plane_bytes, r.lo2[pb], r.hi2[ONE_WORD ? 0 : pb], pb);
        }
    };
    typedef std::conditional_t<WM == 2, u32x2, uint32_t> Staged;
    auto load_stage = [&](int c) -> Staged {
        const uint32_t co = (uint32_t)(PAIR ? min(2 * c, last_first) : c) * plane_bytes;
        if constexpr (WM == 2) return buf_load2(xres, goff, co);
        else return buf_load1(xres, goff, co);
    };
    // the staged piece goes to LDS, the lane's rows come back (LDS serves a wave's accesses in order)
    const uint32_t stage_lane = stage_wave + (uint32_t)lane * 4u;
    auto restage = [&](const Staged &v, Raw &r) {
        if constexpr (WM == 2) *(lds_u32 *)(uintptr_t)stage_lane = __builtin_amdgcn_alignbit(v.y, v.x, gshift);
        else *(lds_u32 *)(uintptr_t)stage_lane = v;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int dy = 0; dy < 3; ++dy) r.lo[pb][dy] = *(lds_cu32 *)(uintptr_t)(loff[pb] + (uint32_t)(dy * SW) * 4u);
    };
    // selectors of the lane's CB channel blocks are contiguous: [step][half][tile][channel in block][block]
    // (QUAD: [step][half][channel of the half][...], two selectors per channel block)
    constexpr int NSEL = QUAD ? 2 * CB : CB;
    const uint32_t sel_step_bytes = (QUAD ? 4u : 2u) * (uint32_t)p.COP * 4u;
    const __amdgpu_buffer_rsrc_t sres = make_rsrc(p.sel, (uint32_t)p.npairs * sel_step_bytes);
    const uint32_t sel_lane = (uint32_t)((QUAD ? 2 * h : h) * p.COP + co0 + n_l * CB) * 4u;
    auto load_sel = [&](int c, uint32_t (&s)[NSEL]) {
        static_assert(CB == 2 || CB == 4, "selector loads are 8 or 16 bytes");
#pragma unroll
        for (int j = 0; j < (QUAD ? 2 : 1); ++j) {
            const uint32_t at = sel_lane + (uint32_t)(j * p.COP) * 4u;
            if constexpr (CB == 4) {
                const u32x4 v = buf_load4(sres, at, (uint32_t)c * sel_step_bytes);
                s[j * CB + 0] = v.x;
                s[j * CB + 1] = v.y;
                s[j * CB + 2] = v.z;
                s[j * CB + 3] = v.w;
            } else {
                const u32x2 v = buf_load2(sres, at, (uint32_t)c * sel_step_bytes);
                s[j * CB + 0] = v.x;
                s[j * CB + 1] = v.y;
            }
        }
    };
    // table rows of the PB pixels -> B operands (24 bytes: 32 FP6 values)
    auto make_B = [&](const Raw &r, v8i (&B)[PB]) {
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            auto window = [&](const uint32_t (&lo)[3], const uint32_t (&hi)[3]) -> uint32_t {
                uint32_t row[3];
#pragma unroll
                for (int dy = 0; dy < 3; ++dy) row[dy] = __builtin_amdgcn_alignbit(ONE_WORD ? lo[dy] : hi[dy], lo[dy], sh[pb]);
                const uint32_t m = m7[pb];
                return (((row[0] & m) | ((row[1] & m) << 3) | ((row[2] & m) << 6)) << lsh[pb]) & vm[pb];
            };
            if constexpr (QUAD) {
                // 16 table values (three words) per channel
                const uint32_t wa = window(r.lo[pb], r.hi[ONE_WORD ? 0 : pb]), wb = window(r.lo2[pb], r.hi2[ONE_WORD ? 0 : pb]);
                const u32x3 qa = *(lds_cu32x3 *)(uintptr_t)(lut_base + wa * MF_LROW);
                const u32x3 qb = *(lds_cu32x3 *)(uintptr_t)(lut_base + wb * MF_LROW);
                B[pb] = (v8i){(int)qa.x, (int)qa.y, (int)qa.z, (int)qb.x, (int)qb.y, (int)qb.z, 0, 0};
                continue;
            }
            uint32_t w;
            if constexpr (ONE) w = (r.lo[pb][0] >> r.byte_shift) & 0xffu;
            else w = window(r.lo[pb], r.hi[ONE_WORD ? 0 : pb]);
            const uint32_t addr = lut_base + w * MF_LROW + (PAIR ? 0u : 32u * (uint32_t)h);
            const u32x4 q0 = *(lds_cu32x4 *)(uintptr_t)addr;
            const u32x2 q1 = *(lds_cu32x2 *)(uintptr_t)(addr + 16);
            B[pb] = (v8i){(int)q0.x, (int)q0.y, (int)q0.z, (int)q0.w, (int)q1.x, (int)q1.y, 0, 0};
        }
    };
    auto make_A = [&](const uint32_t (&s)[NSEL], v8i (&A)[CB]) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const uint32_t sa = s[cb], sb = s[QUAD ? CB + cb : cb];       // QUAD: words 2, 3 come from the second channel's selector
            A[cb] = (v8i){(int)__builtin_amdgcn_perm(0u, 0x00002002u, sa), (int)__builtin_amdgcn_perm(0u, 0x20020000u, sa),
                          (int)__builtin_amdgcn_perm(0x00002002u, 0u, sb), (int)__builtin_amdgcn_perm(0x20020000u, 0u, sb),
                          0, 0, 0, 0};
        }
    };

    v16f acc[CB][PB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;

    // this wave's steps
    const int c_begin = min(split * p.pairs_per_split, p.npairs);
    const int c_end = active ? min(c_begin + p.pairs_per_split, p.npairs) : c_begin;
    const int last = p.npairs - 1;

    // pipeline: memory loads RING steps ahead (a ring of RING register sets: the set of step c is
    // free once its operands exist, which is during step c - 1), operands one step ahead (two
    // sets).  Deeper rings where a step's loads are few registers.  With staging the rows come out of
    // LDS two steps ahead (two sets again, so that no LDS read is waited for in the step that issues
    // it), and the one staged word per step sits in a ring of its own, SRING steps ahead.
    constexpr int RAW_REGS = (STG ? 0 : WM == 3 ? PB + 1 : PB * (WM == 1 ? 3 : 6) * (QUAD ? 2 : 1)) + NSEL;
    constexpr int RING = RAW_REGS <= 16 ? 3 : 2;
    constexpr int SRING = 6;
    constexpr int UNROLL = STG ? 6 : RING % 2 == 0 ? RING : 2 * RING;
    static_assert(UNROLL % RING == 0 && UNROLL % 2 == 0 && (!STG || UNROLL % SRING == 0), "register sets rotate with the unrolled steps");
    Raw raw[STG ? 2 : RING];
    Staged stg[SRING];
    uint32_t sel[RING][NSEL];
    v8i A[2][CB], B[2][PB];
    if constexpr (STG) {
#pragma unroll
        for (int u = 0; u < SRING; ++u) stg[u] = load_stage(min(c_begin + u, last));
    }
#pragma unroll
    for (int u = 0; u < RING; ++u) {
        if constexpr (!STG) load_raw(min(c_begin + u, last), raw[u]);
        load_sel(min(c_begin + u, last), sel[u]);
        __builtin_amdgcn_sched_barrier(0);
    }
    // the table into LDS, the 6 words of every lane half spread to the padded layout
#pragma unroll
    for (int i = 0; i < LUT_WORDS; ++i) {
        const int e = i * (MF_WAVES * 64) + tid;
        const int row = e / (6 * HALVES), rest = e - row * (6 * HALVES);
        const int half = rest / 6, col = rest - 6 * half;
        ((uint32_t *)smem)[row * (MF_LROW / 4) + half * 8 + col] = lutw[i];
    }
    __syncthreads();                               // table visible

    if (c_begin < c_end) {
        if constexpr (STG) {
            restage(stg[0], raw[0]);
            restage(stg[1], raw[1]);
        }
        make_B(raw[0], B[0]);
        make_A(sel[0], A[0]);
        __builtin_amdgcn_sched_barrier(0);
        // One step: the matrix instructions of step c, and between them (the matrix pipe takes ~50
        // cycles per instruction, during which the wave can issue other work) the loads of step
        // c + RING and the operand preparation of step c + 1.  The scheduling groups spell out
        // that interleaving; left alone, the compiler keeps the matrix instructions back to back and
        // moves the loads next to their uses.  u = (c - c_begin) % UNROLL selects the register sets.
        auto step = [&](int c, auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int cur = u % 2, nxt = (u + 1) % 2;
            constexpr int slot_next = (u + 1) % RING, slot_load = u % RING;
            if constexpr (STG) {
                // rows of step c + 2 into the set that held step c's; operands of step c + 1 from the other
                restage(stg[(u + 2) % SRING], raw[cur]);
                stg[u % SRING] = load_stage(min(c + SRING, last));
                load_sel(min(c + RING, last), sel[slot_load]);
                make_B(raw[nxt], B[nxt]);
            } else {
                load_raw(min(c + RING, last), raw[slot_load]);
                load_sel(min(c + RING, last), sel[slot_load]);
                make_B(raw[slot_next], B[nxt]);
            }
            make_A(sel[slot_next], A[nxt]);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)      // (scale operands of zero select the form without block scales)
                    acc[cb][pb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A[cur][cb], B[cur][pb], acc[cb][pb], 4 /* A: FP4 */,
                                                                                  2 /* B: FP6 e2m3 */, 0, 0, 0, 0);
            constexpr int NMF = CB * PB;
            constexpr int NCH = QUAD ? 2 : 1;
            constexpr int NVM = (STG ? 1 : NCH * PB * (WM == 1 || WM == 3 ? 1 : WM == 2 ? 2 : 3)) + NCH;   // loads of a step
            constexpr int NDS = 2 * PB + (STG ? PB * 2 : 0);                     // LDS reads of a step
            constexpr int DS_PER = (NDS + NMF - 1) / NMF;
            constexpr int NVA = NCH * PB * 11 + CB * 4 + 4;                 // vector ALU instructions of a step (estimate)
            constexpr int VM_PER = (NVM + NMF - 1) / NMF, VA_PER = (NVA + NMF - 1) / NMF;
#pragma unroll
            for (int m = 0; m < NMF; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one matrix instruction
                if (STG && m == 0) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // the staged word
                __builtin_amdgcn_sched_group_barrier(0x020, VM_PER, 0);     // loads first: they have the longest way to go
                __builtin_amdgcn_sched_group_barrier(0x002, VA_PER, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, STG ? DS_PER : 2, 0);   // rows and table rows as soon as their addresses exist
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        auto group = [&](int c, auto guarded) {
            // UNROLL consecutive steps; the guarded form (the tail) stops at c_end
            auto run = [&](auto uc) {
                constexpr int u = decltype(uc)::value;
                if (!decltype(guarded)::value || c + u < c_end) step(c + u, uc);
            };
            run(std::integral_constant<int, 0>{});
            run(std::integral_constant<int, 1>{});
            if constexpr (UNROLL > 2) {
                run(std::integral_constant<int, 2>{});
                run(std::integral_constant<int, 3>{});
            }
            if constexpr (UNROLL > 4) {
                run(std::integral_constant<int, 4>{});
                run(std::integral_constant<int, 5>{});
            }
        };
        int c = c_begin;
        for (; c + UNROLL <= c_end; c += UNROLL) group(c, std::false_type{});
        if (c < c_end) group(c, std::true_type{});
    }
    // The {correction, alpha} pairs of the wave's output channels are requested now (the operand
    // registers of the loop are free) and travel during the reduction.
    // The KS waves of a tile share one copy: each fetches a KS-th of it.
    constexpr int FIN_BYTES = 32 * CB * 16 * 8;
    constexpr int FIN_PIECES = FIN_BYTES / 1024;   // of 64 lanes x 16 bytes; 8 or 16, a multiple of KS
    u32x4 finv[FIN_PIECES];
    const int fin_first = split * (FIN_PIECES / KS);
    {
        const u32x4 *src = (const u32x4 *)(p.fin + (size_t)co0 * 16) + fin_first * 64 + lane;
#pragma unroll
        for (int i = 0; i < FIN_PIECES; ++i)
            if (i < FIN_PIECES / KS) finv[i] = src[i * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- partial sums of the KS waves of a tile ---------------------------------------------------------
    // Block q of the tile is finished by the wave with split == q % KS; the other waves pass their
    // partial sums for it through LDS.
    if (KS > 1) {
        constexpr int NPASS = NBLK > 4 ? 2 : 1;    // blocks are reduced NBLK / NPASS at a time to bound the LDS
        constexpr int BPP = NBLK / NPASS;
        // slot of 4 KB: [tile in workgroup][block in pass][writer rank 0 .. KS-2][4 pieces][64 lanes x 16 bytes]
        const uint32_t red_lane = (uint32_t)(uintptr_t)smem + (uint32_t)lane * 16u;
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            __syncthreads();                       // table (or the previous pass) no longer read
#pragma unroll
            for (int ql = 0; ql < BPP; ++ql) {
                const int q = pass * BPP + ql, cb = q / PB, pb = q % PB;
                const int owner = q & (KS - 1);
                if (owner != split) {
                    const int rank = ((split - owner) & (KS - 1)) - 1;
                    const uint32_t a = red_lane + (uint32_t)((((tile_in_wg * BPP + ql) * (KS - 1)) + rank) * 4096);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        u32x4 t;
                        t.x = __float_as_uint(acc[cb][pb][4 * v]);
                        t.y = __float_as_uint(acc[cb][pb][4 * v + 1]);
                        t.z = __float_as_uint(acc[cb][pb][4 * v + 2]);
                        t.w = __float_as_uint(acc[cb][pb][4 * v + 3]);
                        *(lds_u32x4 *)(uintptr_t)(a + v * 1024) = t;
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int ql = 0; ql < BPP; ++ql) {
                const int q = pass * BPP + ql, cb = q / PB, pb = q % PB;
                if ((q & (KS - 1)) == split) {
                    for (int rank = 0; rank < KS - 1; ++rank) {
                        const uint32_t a = red_lane + (uint32_t)((((tile_in_wg * BPP + ql) * (KS - 1)) + rank) * 4096);
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const u32x4 t = *(lds_cu32x4 *)(uintptr_t)(a + v * 1024);
                            acc[cb][pb][4 * v] += __uint_as_float(t.x);
                            acc[cb][pb][4 * v + 1] += __uint_as_float(t.y);
                            acc[cb][pb][4 * v + 2] += __uint_as_float(t.z);
                            acc[cb][pb][4 * v + 3] += __uint_as_float(t.w);
                        }
                    }
                }
            }
        }
    }
    // ---- epilogue: S = 2 M' - fin.x, y = float(S) * alpha ---------------------------------------------
    // The {correction, alpha} pairs of the wave's output channels go through LDS (one 8-byte read
    // per output); stores use a scalar channel offset.  Register r of a block: output channel
    // 8 * (r / 4) + 4 * h + r % 4, pixel n_l.
    __syncthreads();                               // table / partial sums no longer read
    const uint32_t fin_wave = (uint32_t)(uintptr_t)smem + (uint32_t)tile_in_wg * FIN_BYTES;
#pragma unroll
    for (int i = 0; i < FIN_PIECES; ++i)
        if (i < FIN_PIECES / KS) *(lds_u32x4 *)(uintptr_t)(fin_wave + (uint32_t)((fin_first + i) * 64 + lane) * 16u) = finv[i];
    if (KS > 1) __syncthreads();                   // the other waves' parts
    if (!active) return;
    if (p.sign_out) {
        // ---- sign epilogue: bit = ((float)S * alpha + beta >= 0) = (acc * mult >= thr), the next layer's packed rows
        // The 32 lanes of a half hold the pixels of one block of one channel: a ballot turns their signs
        // into a bit string that holds the block's words of that channel (a block is made of whole words,
        // so nobody else writes them and every word gets written).  Lane (c, half) collects word
        // 2 G + half of channel c of the block while the 16 accumulator registers go by (register r is
        // channels cl and cl + 4, in the low and the high half of the ballot), so that a block of 32
        // channels costs one store instruction per pair of words instead of sixteen.
        const int WWo = (g.Wo + 31) / 32;
        const uint32_t oplane = (uint32_t)(g.Ho * WWo);            // words per output channel plane
        const bool short_rows = g.Wo <= 32;
        const int wpb = short_rows ? rows_pb : 1;                  // words of one channel in a block
        const int NG = (wpb + 1) / 2;
        const uint32_t wmask = g.Wo < 32 ? (1u << g.Wo) - 1u : 0xffffffffu;
        const bool takes_hi = (n_l & 4) != 0;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            int n, ho, wo;
            const bool ok = pixel_of(pb, n_l, n, ho, wo);
            // the block's image, its first word inside a channel plane and how many of its words exist (wave-uniform)
            int B = blk0 + pb;
            const bool bvalid = B < p.n_pxblocks;
            if (!bvalid) B = p.n_pxblocks - 1;
            int bn, bword, bwords;
            if (short_rows) {
                bn = B / bpi;
                bword = (B - bn * bpi) * rows_pb;
                bwords = min(rows_pb, g.Ho - bword);
            } else {
                const int R = B / wpr;
                bn = R / g.Ho;
                bword = (R - bn * g.Ho) * WWo + (B - R * wpr);
                bwords = 1;
            }
            if (!bvalid) bwords = 0;
            const unsigned long long okm = __ballot(ok);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int q = cb * PB + pb;
                if (KS > 1 && (q & (KS - 1)) != split) continue;
                const uint32_t fin_lane = fin_wave + (uint32_t)(((cb * 32 + 4 * h) * 16 + ptype[pb]) * 8);
                const int co = co0 + cb * 32 + n_l;                // the channel whose words this lane collects
                if (wpb == 1) {
                    // one word per channel and block (rows longer than 16 pixels): the two halves of the
                    // ballot are the words of channels cl and cl + 4; they go straight into the lanes of
                    // those channels
                    u32x2 f[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) f[r] = *(lds_cu32x2 *)(uintptr_t)(fin_lane + (uint32_t)((8 * (r / 4) + (r % 4)) * 128));
                    uint32_t outw = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int cl = 8 * (r / 4) + (r % 4);
                        const unsigned long long m =
                            __ballot(acc[cb][pb][r] * __uint_as_float(f[r].x) >= __uint_as_float(f[r].y)) & okm;
                        const uint32_t m_lo = (uint32_t)m, m_hi = (uint32_t)(m >> 32);     // wave-uniform
                        asm("v_writelane_b32 %0, %1, %2" : "+v"(outw) : "s"(m_lo), "n"(cl));
                        asm("v_writelane_b32 %0, %1, %2" : "+v"(outw) : "s"(m_hi), "n"(cl + 4));
                    }
                    if (h == 0 && bwords > 0 && co < g.C_out) p.sign_out[(uint32_t)(bn * g.C_out + co) * oplane + (uint32_t)bword] = outw;
                    continue;
                }
                for (int G = 0; G < NG; ++G) {
                    const int j = 2 * G + h;
                    const uint32_t lshift = short_rows ? (uint32_t)(j * g.Wo) & 31u : 0u;
                    uint32_t outw = 0;
                    u32x2 f[16];                                                   // {mult, thr} of the lane's 16 channels
#pragma unroll
                    for (int r = 0; r < 16; ++r) f[r] = *(lds_cu32x2 *)(uintptr_t)(fin_lane + (uint32_t)((8 * (r / 4) + (r % 4)) * 128));
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int cl = 8 * (r / 4) + (r % 4);                      // channel inside the block, lane half 0
                        const unsigned long long m =
                            __ballot(acc[cb][pb][r] * __uint_as_float(f[r].x) >= __uint_as_float(f[r].y)) & okm;
                        const uint32_t src = takes_hi ? (uint32_t)(m >> 32) : (uint32_t)m;
                        if ((n_l & ~4) == cl) outw = (src >> lshift) & wmask;
                    }
                    if (j < bwords && co < g.C_out) p.sign_out[(uint32_t)(bn * g.C_out + co) * oplane + (uint32_t)(bword + j)] = outw;
                }
            }
        }
        return;
    }
    const __amdgpu_buffer_rsrc_t yres = make_rsrc(p.y, (uint32_t)((size_t)g.N * g.C_out * g.HoWo * 4u));
    const uint32_t chan_bytes = (uint32_t)g.HoWo * 4u;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int q = cb * PB + pb;
            if (KS > 1 && (q & (KS - 1)) != split) continue;
            const uint32_t fin_lane = fin_wave + (uint32_t)(((cb * 32 + 4 * h) * 16 + ptype[pb]) * 8);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cs = co0 + cb * 32 + 8 * (r / 4) + (r % 4);          // wave-uniform part of the channel
                const u32x2 f = *(lds_cu32x2 *)(uintptr_t)(fin_lane + (uint32_t)((8 * (r / 4) + (r % 4)) * 128));
                const float v = (float)(2 * (int)acc[cb][pb][r] - (int)f.x) * __uint_as_float(f.y);
                if (cs + 4 * h < g.C_out) buf_store(yres, v, yoff[pb], (uint32_t)cs * chan_bytes);
            }
        }
}

template <int PB, int CB, int WM, bool PAIR, bool STG, bool QUAD = false>
__global__ __launch_bounds__(MF_WAVES * 64, 2)
void subbit_mfma_kernel(const MfParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    mf_tile_body<PB, CB, WM, PAIR, STG, QUAD>(p, blockIdx.x, smem);
}

// Several layers in ONE launch: workgroups [first_block[l], first_block[l + 1]) run layer l.  The
// layers of a stack that do not depend on each other (each has its own input) then share the
// chip: no launch ends with a few busy compute units, and while the workgroups of one layer store
// their outputs those of the next are in their matrix loops.  Only the forms the default plan picks
// for subsets of up to 32 members are compiled in (`variant`, see mf_many_variant).
constexpr int MF_MANY_MAX = 16;
struct MfManyParams {
    int n_layers;
    int first_block[MF_MANY_MAX + 1];
    int variant[MF_MANY_MAX];
    MfParams layer[MF_MANY_MAX];
};

__global__ __launch_bounds__(MF_WAVES * 64, 2)
void subbit_mfma_many_kernel(const MfManyParams pm)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int b = blockIdx.x;
    int l = 0;
    while (l + 1 < pm.n_layers && b >= pm.first_block[l + 1]) ++l;      // block-uniform
    const MfParams &p = pm.layer[l];
    const unsigned block = (unsigned)(b - pm.first_block[l]);
    switch (pm.variant[l]) {
    case 0: mf_tile_body<4, 2, 0, true, false>(p, block, smem); break;
    case 1: mf_tile_body<4, 2, 1, true, false>(p, block, smem); break;
    case 2: mf_tile_body<4, 2, 2, true, false>(p, block, smem); break;
    case 3: mf_tile_body<4, 2, 1, true, true>(p, block, smem); break;
    case 4: mf_tile_body<4, 2, 2, true, true>(p, block, smem); break;
    case 5: mf_tile_body<2, 4, 0, true, false>(p, block, smem); break;
    case 6: mf_tile_body<2, 4, 1, true, false>(p, block, smem); break;
    default: mf_tile_body<2, 4, 2, true, false>(p, block, smem); break;
    }
}

// ---- host side -------------------------------------------------------------------------------------


template <int PB, int CB, int WM, bool PAIR, bool STG, bool QUAD = false>
int launch_mf_one(const MfPlan &pl, const MfParams &prm, hipStream_t s)
{
    auto kern = subbit_mfma_kernel<PB, CB, WM, PAIR, STG, QUAD>;
    static LdsGrant grant;
    if (grant_dynamic_lds((const void *)kern, pl.lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)pl.n_wgs), dim3(MF_WAVES * 64), pl.lds, s, prm);
    return check_launch();
}

template <int PB, int CB, bool PAIR>
int launch_mf_pair(const MfPlan &pl, const MfParams &prm, hipStream_t s)
{
    if (pl.one) return launch_mf_one<PB, CB, 3, PAIR, false>(pl, prm, s);
    if (prm.g.WW == 1) return pl.stage ? launch_mf_one<PB, CB, 1, PAIR, true>(pl, prm, s) : launch_mf_one<PB, CB, 1, PAIR, false>(pl, prm, s);
    if (prm.g.WW == 2) return pl.stage ? launch_mf_one<PB, CB, 2, PAIR, true>(pl, prm, s) : launch_mf_one<PB, CB, 2, PAIR, false>(pl, prm, s);
    return launch_mf_one<PB, CB, 0, PAIR, false>(pl, prm, s);
}

template <int PB, int CB>
int launch_mf_quad(const MfPlan &pl, const MfParams &prm, hipStream_t s)
{
    if (prm.g.WW == 1) return launch_mf_one<PB, CB, 1, true, false, true>(pl, prm, s);
    if (prm.g.WW == 2) return launch_mf_one<PB, CB, 2, true, false, true>(pl, prm, s);
    return launch_mf_one<PB, CB, 0, true, false, true>(pl, prm, s);
}

template <int PB, int CB>
int launch_mf(const MfPlan &pl, const MfParams &prm, hipStream_t s)
{
    if (pl.quad) return launch_mf_quad<PB, CB>(pl, prm, s);
    return pl.pair ? launch_mf_pair<PB, CB, true>(pl, prm, s) : launch_mf_pair<PB, CB, false>(pl, prm, s);
}

}  // namespace

bool subbit_mfma_supported(const Geom &g)
{
    // 64 contraction slots per matrix instruction: two input channels of up to 32 subset members or
    // one of up to 64; 32-bit byte offsets into the packed input, the selector table and the output
    const int64_t x_words = (int64_t)g.N * g.C_in * g.H * g.WW;
    const int64_t sel_words = (int64_t)2 * (g.C_in + 1) * (g.C_out + 127);
    const int64_t y_words = (int64_t)g.P * g.C_out;
    return g.K <= 64 && (g.K > 32 || g.C_in >= 2) && x_words < ((int64_t)1 << 30) && sel_words < ((int64_t)1 << 30) &&
           y_words < ((int64_t)1 << 30) && g.P < ((int64_t)1 << 31) - 4096;
}

int subbit_mfma_slots_per_channel(const Geom &g)
{
    const MfPlan pl = mf_plan(g, false);
    return pl.quad ? 16 : pl.pair ? 32 : 64;
}

// The plain and the sign-epilogue form cut the pixels into blocks differently and may therefore split
// the input channels differently (and, for small subsets, pick different table layouts): the size
// covers both, so that one workspace serves every entry point of a layer.
size_t subbit_mfma_workspace_bytes(const Geom &g)
{
    const size_t a = mf_plan(g, false).bytes, b = mf_plan(g, true).bytes;
    return a > b ? a : b;
}

namespace {

MfParams mf_params(const MfPlan &pl, const Geom &g, const void *x, float *y, void *ws, const SignEpilogue *sign)
{
    MfParams prm;
    prm.x = (const uint32_t *)x;
    prm.sel = (const uint32_t *)((char *)ws + pl.off_sel);
    prm.fin = (const uint2 *)((char *)ws + pl.off_fin);
    prm.lut = (const uint32_t *)((char *)ws + pl.off_lut);
    prm.y = y;
    prm.sign_out = sign ? sign->out : nullptr;
    prm.g = g;
    prm.COP = pl.COP;
    prm.KS = pl.KS;
    prm.npairs = pl.npairs;
    prm.pairs_per_split = (pl.npairs + pl.KS - 1) / pl.KS;
    prm.n_cotiles = pl.n_cotiles;
    prm.n_tiles = pl.n_tiles;
    prm.n_pxblocks = (int)pl.n_pxblocks;
    prm.x_bytes = 0;
    prm.cw_bytes = 0;
    return prm;
}

int launch_mf_conv(const MfPlan &pl, const MfParams &prm, hipStream_t s)
{
    const MfCfg &c = pl.cfg;
    if (c.PB == 4 && c.CB == 2) return launch_mf<4, 2>(pl, prm, s);
    if (c.PB == 2 && c.CB == 4) return launch_mf<2, 4>(pl, prm, s);
    if (c.PB == 2 && c.CB == 2) return launch_mf<2, 2>(pl, prm, s);
    if (c.PB == 1 && c.CB == 4) return launch_mf<1, 4>(pl, prm, s);
    if (c.PB == 1 && c.CB == 2) return launch_mf<1, 2>(pl, prm, s);
    return SNN_ERR_UNSUPPORTED;
}

StackTables stack_tables(const MfPlan &pl, void *ws)
{
    StackTables st;
    st.negcorr = (int16_t *)((char *)ws + pl.off_negcorr);
    st.alphap = (float *)((char *)ws + pl.off_alphap);
    st.sched = (uint32_t *)((char *)ws + pl.off_sched);
    st.COP = pl.COP;
    return st;
}

WeightParams weight_params(const MfPlan &pl, const Geom &g, const MfParams &prm, const float *w, const uint16_t *codebook,
                           const float *alpha, const float *beta, uint16_t *idx_out)
{
    WeightParams wp;
    wp.w = w;
    wp.codebook = codebook;
    wp.alpha = alpha;
    wp.beta = beta;
    wp.idx_out = idx_out;
    wp.sel = (uint32_t *)prm.sel;
    wp.fin = (uint2 *)prm.fin;
    wp.lut = (uint32_t *)prm.lut;
    wp.C_in = g.C_in;
    wp.C_out = g.C_out;
    wp.COP = pl.COP;
    wp.CB = pl.cfg.CB;
    wp.K = g.K;
    wp.pair = pl.quad ? 2 : pl.pair ? 1 : 0;
    wp.lut_blocks = (512 * (pl.pair ? 6 : 12) + 255) / 256;
    wp.st = stack_tables(pl, (char *)prm.sel - pl.off_sel);
    return wp;
}

}  // namespace

// Weights-side work of several layers in one launch (groups of PREP_MANY_MAX); every layer must be one
// the matrix-core kernel takes.  beta[l] non-null: thresholds for the sign epilogue.
int launch_subbit_prepare_many(int n_layers, const Geom *gs, const float *const *w, const uint16_t *const *codebook,
                               const float *const *alpha, const float *const *beta, uint16_t *const *idx_out,
                               void *const *ws, hipStream_t s)
{
    for (int l0 = 0; l0 < n_layers; l0 += PREP_MANY_MAX) {
        PrepManyParams pm;
        pm.n_layers = n_layers - l0 < PREP_MANY_MAX ? n_layers - l0 : PREP_MANY_MAX;
        int64_t blocks = 0;
        for (int i = 0; i < pm.n_layers; ++i) {
            const int l = l0 + i;
            const bool sign = beta[l] != nullptr;
            const MfPlan pl = mf_plan(gs[l], sign);
            if (pl.n_wgs > 0x7fffffffLL || pl.lds > 160 * 1024 || pl.n_pxblocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
            const MfParams prm = mf_params(pl, gs[l], nullptr, nullptr, ws[l], nullptr);
            pm.layer[i] = weight_params(pl, gs[l], prm, w[l], codebook[l], alpha[l], beta[l], idx_out[l]);
            pm.first_block[i] = (int)blocks;
            blocks += pl.COP + pm.layer[i].lut_blocks;
            if (blocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
        }
        pm.first_block[pm.n_layers] = (int)blocks;
        for (int i = pm.n_layers + 1; i <= PREP_MANY_MAX; ++i) pm.first_block[i] = (int)blocks;
        hipLaunchKernelGGL(subbit_prepare_many_kernel, dim3((unsigned)blocks), dim3(256), 0, s, pm);
        const int rc = check_launch();
        if (rc != SNN_OK) return rc;
    }
    return SNN_OK;
}

int launch_subbit_mfma(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                       const float *alpha, float *y, void *ws, hipStream_t s, const SignEpilogue *sign, int phases, int tau)
{
    const MfPlan pl = mf_plan(g, sign != nullptr);
    if (pl.n_wgs > 0x7fffffffLL || pl.lds > 160 * 1024 || pl.n_pxblocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
    const MfParams prm = mf_params(pl, g, x, y, ws, sign);

    const int sel_blocks = (pl.COP / 32) * ((g.C_in + 31) / 32);
    const int corr_blocks = (pl.COP + 3) / 4;
    const int lut_blocks = (512 * (pl.pair ? 6 : 12) + 255) / 256;
    if (phases & SNN_PHASE_PREPARE)
        hipLaunchKernelGGL(subbit_mfma_prep_kernel, dim3((unsigned)(sel_blocks + corr_blocks + lut_blocks)), dim3(256), 0, s,
                           codebook, (const void *)idx, tau, g.C_in, g.C_out, pl.COP, pl.cfg.CB, g.K, pl.quad ? 2 : pl.pair ? 1 : 0, sel_blocks, lut_blocks, alpha,
                           (uint32_t *)prm.sel, (uint2 *)prm.fin, (uint32_t *)prm.lut, sign ? sign->beta : nullptr, 9, stack_tables(pl, ws));
    if (!(phases & SNN_PHASE_CONVOLVE)) return check_launch();
    return launch_mf_conv(pl, prm, s);
}

// The convolutions of several prepared layers (fp32 output).  Layers whose plan is one of the forms
// compiled into subbit_mfma_many_kernel share launches of up to MF_MANY_MAX layers; any other layer
// gets a launch of its own.
namespace {

int mf_many_variant(const MfPlan &pl, const Geom &g)
{
    if (pl.one || pl.quad || !pl.pair) return -1;
    const int wm = g.WW <= 2 ? g.WW : 0;
    if (pl.cfg.PB == 4 && pl.cfg.CB == 2) return pl.stage ? (wm == 1 ? 3 : 4) : wm;
    if (pl.cfg.PB == 2 && pl.cfg.CB == 4 && !pl.stage) return 5 + wm;
    return -1;
}

}  // namespace

int launch_subbit_mfma_many(int n_layers, const Geom *gs, const void *const *x, float *const *y, void *const *ws, hipStream_t s)
{
    static LdsGrant grant;
    MfManyParams pm;
    pm.n_layers = 0;
    int64_t blocks = 0;
    size_t lds = 0;
    auto flush = [&]() -> int {
        if (pm.n_layers == 0) return SNN_OK;
        pm.first_block[pm.n_layers] = (int)blocks;
        for (int i = pm.n_layers + 1; i <= MF_MANY_MAX; ++i) pm.first_block[i] = (int)blocks;
        if (grant_dynamic_lds((const void *)subbit_mfma_many_kernel, lds, grant) != SNN_OK) return SNN_ERR_LAUNCH;
        hipLaunchKernelGGL(subbit_mfma_many_kernel, dim3((unsigned)blocks), dim3(MF_WAVES * 64), lds, s, pm);
        pm.n_layers = 0;
        blocks = 0;
        lds = 0;
        return check_launch();
    };
    // In a shared launch the split of the input channels over waves is chosen for the length of a wave's
    // run (about 64 steps: measured best on the ResNet-18 stack), not to fill the chip with one layer.
    const int target_steps = 64;
    for (int l = 0; l < n_layers; ++l) {
        MfPlan pl = mf_plan(gs[l]);
        {
            int ks = 1;
            while (ks < 4 && pl.npairs / (2 * ks) >= target_steps) ks *= 2;
            pl.KS = ks;
            pl.n_wgs = (pl.n_tiles * ks + MF_WAVES - 1) / MF_WAVES;
            const int nblk = pl.cfg.PB * pl.cfg.CB;
            const size_t lut_bytes = (size_t)512 * mf_lrow(pl.pair) + (pl.stage ? (size_t)MF_WAVES * MF_STAGE_BYTES : 0);
            const size_t red_bytes = ks > 1 ? (size_t)(MF_WAVES / ks) * (nblk > 4 ? nblk / 2 : nblk) * (ks - 1) * 4096 : 0;
            const size_t fin_bytes = (size_t)MF_WAVES * 32 * pl.cfg.CB * 16 * 8;
            pl.lds = lut_bytes > red_bytes ? lut_bytes : red_bytes;
            if (fin_bytes > pl.lds) pl.lds = fin_bytes;
        }
        if (pl.n_wgs > 0x7fffffffLL || pl.lds > 160 * 1024 || pl.n_pxblocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
        const MfParams prm = mf_params(pl, gs[l], x[l], y[l], ws[l], nullptr);
        const int variant = mf_many_variant(pl, gs[l]);
        if (variant < 0 || blocks + pl.n_wgs > 0x7fffffffLL) {
            int rc = flush();
            if (rc != SNN_OK) return rc;
            if (variant < 0) {
                rc = launch_mf_conv(pl, prm, s);
                if (rc != SNN_OK) return rc;
                continue;
            }
        }
        pm.layer[pm.n_layers] = prm;
        pm.variant[pm.n_layers] = variant;
        pm.first_block[pm.n_layers] = (int)blocks;
        blocks += pl.n_wgs;
        if (pl.lds > lds) lds = pl.lds;
        if (++pm.n_layers == MF_MANY_MAX) {
            const int rc = flush();
            if (rc != SNN_OK) return rc;
        }
    }
    return flush();
}

// Alg. 1 forward of a layer in two launches: the front kernel (projection, selector / finishing /
// lookup tables, and sign + packing of x into `xr` unless x is null: then `xr` holds the packed
// input already), then the convolution on `xr`, ending in y or in the sign epilogue.
int launch_subbit_forward_mfma(const Geom &g, const float *x, const float *w, const uint16_t *codebook,
                               const float *alpha, uint16_t *idx_out, float *y, uint32_t *xr, void *ws, hipStream_t s,
                               const SignEpilogue *sign)
{
    const MfPlan pl = mf_plan(g, sign != nullptr);
    if (pl.n_wgs > 0x7fffffffLL || pl.lds > 160 * 1024 || pl.n_pxblocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
    const MfParams prm = mf_params(pl, g, xr, y, ws, sign);

    FrontParams fp;
    fp.x = x;
    fp.xr = xr;
    fp.rows = (int64_t)g.N * g.C_in * g.H;
    fp.W = g.W;
    fp.WW = g.WW;
    const PackRowsPlan pk = pack_rows_plan(x, fp.rows, g.W);
    fp.rows_per_block = pk.rows_per_block;
    fp.vec = pk.vec;
    fp.pack_blocks = x ? pk.blocks : 0;
    fp.wp = weight_params(pl, g, prm, w, codebook, alpha, sign ? sign->beta : nullptr, idx_out);
    const int64_t blocks = (int64_t)pl.COP + fp.wp.lut_blocks + fp.pack_blocks;
    if (blocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(subbit_front_kernel, dim3((unsigned)blocks), dim3(256), 0, s, fp);
    return launch_mf_conv(pl, prm, s);
}

// ---- 1x1 layers (the extension to bottleneck blocks: vectors of 8 input channels) -----------------------------
// The same kernel with the byte of 8 channel signs as the window; `g` is the real layer, the kernel sees
// C_in / 8 groups as its input channels.
namespace {

Geom groups_geom(const Geom &g)
{
    Geom gk = g;
    gk.C_in = g.C_in / 8;
    return gk;
}

}  // namespace

bool subbit_conv1x1_supported(const Geom &g)
{
    const int G = g.C_in / 8;
    const int64_t x_words = (int64_t)g.N * g.H * g.W * g.CW;
    const int64_t sel_words = (int64_t)2 * (G + 1) * (g.C_out + 127);
    const int64_t y_words = (int64_t)g.P * g.C_out;
    return g.C_in % 8 == 0 && g.K <= 64 && (g.K > 32 || G >= 2) && x_words < ((int64_t)1 << 30) && sel_words < ((int64_t)1 << 30) &&
           y_words < ((int64_t)1 << 30) && g.P < ((int64_t)1 << 31) - 4096;
}

size_t subbit_conv1x1_workspace_bytes(const Geom &g) { return mf_plan(groups_geom(g), false, true).bytes; }

int launch_subbit_conv1x1(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx, const float *alpha,
                          float *y, void *ws, hipStream_t s, int phases)
{
    const Geom gk = groups_geom(g);
    const MfPlan pl = mf_plan(gk, false, true);
    if (pl.n_wgs > 0x7fffffffLL || pl.lds > 160 * 1024 || pl.n_pxblocks > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
    MfParams prm = mf_params(pl, gk, x, y, ws, nullptr);
    prm.cw_bytes = (uint32_t)g.CW * 4u;
    prm.x_bytes = (uint32_t)((size_t)g.N * g.H * g.W * g.CW * 4u);
    const int sel_blocks = (pl.COP / 32) * ((gk.C_in + 31) / 32);
    const int corr_blocks = (pl.COP + 3) / 4;
    const int lut_blocks = (256 * (pl.pair ? 6 : 12) + 255) / 256;
    if (phases & SNN_PHASE_PREPARE)
        hipLaunchKernelGGL(subbit_mfma_prep_kernel, dim3((unsigned)(sel_blocks + corr_blocks + lut_blocks)), dim3(256), 0, s, codebook,
                           (const void *)idx, 0, gk.C_in, g.C_out, pl.COP, pl.cfg.CB, g.K, pl.pair ? 1 : 0, sel_blocks, lut_blocks, alpha,
                           (uint32_t *)prm.sel, (uint2 *)prm.fin, (uint32_t *)prm.lut, (const float *)nullptr, 8, stack_tables(pl, ws));
    if (!(phases & SNN_PHASE_CONVOLVE)) return check_launch();
    return launch_mf_conv(pl, prm, s);
}

// ---- tau-bit index storage (Sec. 4.4 / Fig. 5) ---------------------------------------------------------------
namespace {

// one thread per 32-bit word of the bit stream: it collects the indices that overlap its word
__global__ __launch_bounds__(256)
void pack_indices_kernel(const uint16_t *__restrict__ idx, int64_t n, int tau, uint32_t *__restrict__ out, int64_t words)
{
    const int64_t wd = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (wd >= words) return;
    const int64_t bit0 = wd * 32;
    uint32_t v = 0;
    for (int64_t i = bit0 / tau; i < n && i * tau < bit0 + 32; ++i) {
        const int64_t at = i * tau - bit0;               // position of the index's bit 0 in this word
        const uint32_t k = (uint32_t)idx[i] & ((1u << tau) - 1u);
        v |= at >= 0 ? k << at : k >> -at;
    }
    out[wd] = v;
}

}  // namespace

int launch_pack_indices(const uint16_t *idx, int64_t n, int tau, uint32_t *out, hipStream_t s)
{
    const int64_t words = (n * tau + 31) / 32;
    const int64_t blocks = (words + 255) / 256;
    if (blocks > 0x7fffffffLL) return SNN_ERR_INVALID_ARG;
    if (blocks > 0) hipLaunchKernelGGL(pack_indices_kernel, dim3((unsigned)blocks), dim3(256), 0, s, idx, n, tau, out, words);
    return check_launch();
}

}  // namespace snn
