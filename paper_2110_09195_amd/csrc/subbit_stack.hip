// Sub-bit 3x3 convolutions (Sec. 4.5 / Fig. 6) of a STACK of prepared layers in one launch of resident
// workers.
//
// The arithmetic is that of subbit_mfma.hip: stage 1 is a lookup of the 9-bit window in a 512-row
// table of match counts m_k - 4 (FP6), stage 2 the product of that row with the one-hot row (FP4) of
// every output channel's index, two input channels per v_mfma_f32_32x32x64_f8f6f4, exact fp32
// sums; S = 2 M - correction(channel, border type), y = float(S) * alpha.  What differs is how the
// work reaches the chip:
//   * a worker is ONE wave (a workgroup of 64 lanes) that stays resident and takes (layer, tile)
//     items from a counter in device memory until none is left: no launch ends with a few busy
//     compute units, a wave that stores its outputs shares its SIMD with one that multiplies, and
//     items are handed out longest first so that the last ones are short;
//   * everything a wave needs is private to it - its copy of the layer's table (12 KB of LDS, kept
//     while the layer does not change), the staged input rows, the finishing tables of its channels -
//     so no wave ever waits for another (no barriers, no partial sums to exchange: a tile always runs
//     over all input channels);
//   * the finishing step reads {correction, alpha} of four consecutive channels with one LDS access
//     from tables the wave loaded at the start of the tile (border type major), and turns the
//     accumulator into the output with one fused multiply-add and one multiply.
// Only the forms the default plan picks for subsets of up to 32 members are here (two input
// channels per instruction, fp32 output); everything else goes through subbit_mfma.hip.
#include "subbit_mfma_plan.h"

#include <algorithm>
#include <type_traits>
#include <utility>
#include <vector>

namespace snn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const u32x4 lds_cu32x4;
typedef __attribute__((address_space(3))) const u32x2 lds_cu32x2;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) const uint32_t lds_cu32;
typedef __attribute__((address_space(3))) uint32_t lds_u32;

constexpr int ST_MAX_LAYERS = 16;
constexpr int ST_MAX_RUNS = 64;
constexpr int ST_WORKERS_PER_CU = 8;           // two waves per SIMD: 256 vector registers each
constexpr uint32_t ST_QUEUES = MF_SCHED_QUEUES; // item queues: one per XCD
constexpr uint32_t ST_GROUP_LOG2 = 4, ST_GROUP = 1u << ST_GROUP_LOG2;      // consecutive items a queue owns at a time

// LDS of a worker
// The table (row = window, 32 FP6 values = 24 bytes) is kept as two arrays, the first 16 bytes of every row and
// the last 8: a row is then one 16-byte and one 8-byte read at their natural alignment, which the LDS serves
// in two thirds of the time of three 8-byte reads of a 24-byte row (random rows: bank conflicts).
constexpr int ST_LUT8_OFF = 512 * 16;
constexpr int ST_LUT_BYTES = 512 * 24;
constexpr int ST_STAGE_OFF = ST_LUT_BYTES;
constexpr int ST_ALPHA_OFF = ST_STAGE_OFF + MF_STAGE_BYTES;    // float [128]
constexpr int ST_CORR_OFF = ST_ALPHA_OFF + 128 * 4;            // int16 [16][32 CB]
constexpr int ST_RUNS_OFF = ST_CORR_OFF + 16 * 128 * 2;        // {first item, first tile | layer << 24} of the 64 runs
constexpr int ST_LDS_BYTES = ST_RUNS_OFF + ST_MAX_RUNS * 8;
static_assert(ST_ALPHA_OFF % 16 == 0 && ST_CORR_OFF % 16 == 0 && ST_RUNS_OFF % 8 == 0, "aligned LDS accesses");
static_assert(ST_WORKERS_PER_CU * ST_LDS_BYTES <= 160 * 1024, "all workers of a compute unit fit its LDS");

// Division by a divisor fixed per layer (1 <= d < 2^31) of numerators below 2^31: q = mulhi(n, mul) >> shift with
// mul = floor(2^(31 + s) / d) + 1, s = ceil(log2 d), shift = s - 1 (exact: mul * d - 2^(31 + s) is in (0, 2^s]);
// d = 1 is mul = 0.  The kernel's per-tile set-up is a dozen divisions by H_out * W_out, W_out, H and the
// number of channel tiles; the generic sequence costs forty instructions each.
struct Divisor {
    uint32_t mul, shift;
};

inline Divisor make_divisor(uint32_t d)
{
    if (d <= 1u) return {0u, 0u};
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    return {(uint32_t)((1ull << (31 + s)) / d) + 1u, s - 1u};
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const Divisor &d)
{
    return d.mul ? __umulhi(n, d.mul) >> d.shift : n;
}

struct StackLayer {
    const uint32_t *x;        // packed rows [N][C_in][H][WW]
    const uint32_t *lut;      // table images: [512][6] words (row = window, 32 FP6 values m_k - 4), then the split image
    const uint32_t *sel;      // [steps][2][COP] selector words of the one-hot operand
    const int16_t *negcorr;   // [16][COP]: -(2 corr + C_in (valid_taps - 8)) per (border type, output channel)
    const float *alpha;       // [COP]
    float *y;
    int N, C_in, C_out, H, W, stride, Ho, Wo, HoWo, WW, P;
    int COP, npairs, n_cotiles, n_pxblocks;
    int variant;
    Divisor div_HoWo, div_Wo, div_H, div_cotiles;
};

// Items [run_first_item[r], run_first_item[r + 1]) are tiles run_first_tile[r] ... of layer run_layer[r].
struct StackParams {
    uint32_t *sched;          // MF_SCHED_WORDS words: a draw counter per queue (MF_SCHED_STRIDE apart), workers that have left; all zero before and after a launch
    int n_runs, n_items, n_workers;
    int n_matrix_items;       // items are dealt from two lists in proportion: [0, n_matrix_items) and the rest of the run table
    uint32_t deal_ratio;      // ceil(2^32 * second list / dealt items); 0: one list only
    int n_tail;               // the last n_tail items are the last n_tail entries of the first list, not dealt
    int run_first_item[ST_MAX_RUNS + 1];
    int run_first_tile[ST_MAX_RUNS];
    unsigned char run_layer[ST_MAX_RUNS];
    StackLayer layer[ST_MAX_LAYERS];
};


template <int... I, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// One tile: PB blocks of 32 pixels x CB blocks of 32 output channels, all input channels.
// WM: words per packed row (1, 2; 0 for wider rows).  STG: the packed rows the tile touches are few
// enough that ONE load per step brings them all (lane s of a half: piece s of the run of rows that
// starts at the first pixel's top row); they pass through the wave's piece of LDS and every lane
// reads one 32-bit piece per window row from there.
template <int PB, int CB, int WM, bool STG>
__device__ __forceinline__ void stack_tile(const StackLayer &layer, const int tile, const uint32_t lds0, const bool new_layer,
                                           uint32_t *const sched, uint32_t &drawn)
{
    const StackLayer &L = layer;
    static_assert(!STG || WM == 1 || WM == 2, "staging needs rows that are consecutive in memory");
    constexpr int NCH = 32 * CB;
    // (the lane number is made opaque here and again before the finishing step: what is derived from it is
    // then computed where it is used instead of being carried, in registers the loop needs, from the
    // start of the kernel)
    int lane = threadIdx.x;
    asm volatile("" : "+v"(lane));
    const int n_l = lane & 31, h = lane >> 5;
    const int px_tile = (int)fast_div((uint32_t)tile, L.div_cotiles);
    const int co_tile = tile - px_tile * L.n_cotiles;
    const int blk0 = px_tile * PB;                 // first pixel block of the tile
    const int co0 = co_tile * NCH;

    // Requested first, stored to LDS once the loop's first loads are under way: the layer's table if the
    // worker's last tile belonged to another layer (the split image: 768 pieces of 16 bytes, copied as they
    // are), and the finishing tables of the tile's channels.
    constexpr int CR = NCH / 8;                    // 16-byte pieces of the correction table per border type
    constexpr int CROUNDS = 16 * CR / 64;
    u32x4 lut_t[12], tab_a = {0u, 0u, 0u, 0u}, tab_c[CROUNDS];
    if (new_layer) {
#pragma unroll
        for (int i = 0; i < 12; ++i) lut_t[i] = ((const u32x4 *)(L.lut + MF_LUT_SPLIT_WORDS))[i * 64 + lane];
    }
    if (lane < NCH / 4) tab_a = ((const u32x4 *)(L.alpha + co0))[lane];
#pragma unroll
    for (int q = 0; q < CROUNDS; ++q) {
        const int e = q * 64 + lane, type = e / CR, pc = e - type * CR;
        tab_c[q] = *(const u32x4 *)(L.negcorr + (size_t)type * L.COP + co0 + pc * 8);
    }
    constexpr int RAW_REGS = (STG ? 0 : PB * (WM == 1 ? 3 : 6)) + CB;
    constexpr int RING = !STG && PB <= 2 && RAW_REGS <= 14 ? 3 : 2;
    // selectors of the lane's CB channel blocks are contiguous: [step][half][tile][channel in block][block]
    const uint32_t sel_step_bytes = 2u * (uint32_t)L.COP * 4u;
    const __amdgpu_buffer_rsrc_t sres = make_rsrc(L.sel, (uint32_t)L.npairs * sel_step_bytes);
    const uint32_t sel_lane = (uint32_t)(h * L.COP + co0 + n_l * CB) * 4u;
    auto load_sel = [&](int c, uint32_t (&s)[CB]) {
        static_assert(CB == 2 || CB == 4, "selector loads are 8 or 16 bytes");
        if constexpr (CB == 4) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(sres, (int)sel_lane, (int)((uint32_t)c * sel_step_bytes), 0);
            s[0] = v.x;
            s[1] = v.y;
            s[2] = v.z;
            s[3] = v.w;
        } else {
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(sres, (int)sel_lane, (int)((uint32_t)c * sel_step_bytes), 0);
            s[0] = v.x;
            s[1] = v.y;
        }
    };
    // the selector words of the first steps depend on nothing but the tile's channels: requested before the
    // window geometry is worked out, they arrive while it is
    const int last = L.npairs - 1;
    uint32_t sel[RING][CB];
#pragma unroll
    for (int u = 0; u < RING; ++u) load_sel(min(u, last), sel[u]);
    __builtin_amdgcn_sched_barrier(0);

    // ---- per-lane window geometry of the PB pixels (pixel n_l of every block) ----------------------
    // Block B is pixels 32 B .. 32 B + 31 of the flattened (n, ho, wo) order; lanes past the end work
    // on the last pixel and are not written.
    auto pixel_of = [&](int pb, int lane_px, int &n, int &ho, int &wo) -> bool {
        int B = blk0 + pb;
        bool ok = B < L.n_pxblocks;
        if (!ok) B = L.n_pxblocks - 1;
        int pp = B * 32 + lane_px;
        if (pp >= L.P) {
            ok = false;
            pp = L.P - 1;
        }
        n = (int)fast_div((uint32_t)pp, L.div_HoWo);
        const int r = pp - n * L.HoWo;
        ho = (int)fast_div((uint32_t)r, L.div_Wo);
        wo = r - ho * L.Wo;
        return ok;
    };
    // This lane looks at input channel (2 c + h) in step c.  It loads three consecutive packed rows
    // starting at row max(hc - 1, 0), words (jlo, jlo + 1), and cuts row dy of the window out of the
    // 64-bit string {hi, lo} at bit `sh`.  Two cases are folded into a final shift `lsh` of the 9-bit
    // window so that no load starts before the tensor: top image row (the rows loaded are window rows
    // 1, 2, 3: shift by 3) and first image column (the bits cut out are columns 0, 1, 2: keep two,
    // shift by 1).  Words from outside the row, the image or the tensor (read as zero) only reach
    // window bits whose taps lie outside the image, and `vm` masks those off.
    const uint32_t plane_bytes = (uint32_t)(L.H * L.WW) * 4u;
    uint32_t xoff[PB], sh[PB], wd[PB], wmul[PB], vm[PB], yoff[PB], loff[PB];
    int ptype[PB];
    const uint32_t stage_wave = lds0 + ST_STAGE_OFF;
    constexpr int SW = WM == 2 ? 3 : 1;            // pieces per staged row
    int R_first = 0;
    uint32_t goff = 0xffffffffu;                   // byte offset of the word(s) this lane stages (channel h of the step)
    uint32_t gshift = 0;
    if constexpr (STG) {
        int n0, ho0, wo0;
        pixel_of(0, 0, n0, ho0, wo0);              // the tile's first pixel (wave-uniform)
        const int hc0 = ho0 * L.stride;
        R_first = n0 * L.H + (hc0 == 0 ? 0 : hc0 - 1);
        const int R = R_first + n_l / SW, piece = n_l % SW;
        const int n = (int)fast_div((uint32_t)R, L.div_H), hr = R - n * L.H;
        if (n < L.N) goff = (uint32_t)(((n * L.C_in + h) * L.H + hr) * L.WW + (piece == 2 ? 1 : 0)) * 4u;
        gshift = piece == 1 ? 16u : 0u;
    }
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(L.x, (uint32_t)L.N * (uint32_t)L.C_in * plane_bytes);
    // step c -> first channel of the pair (the last step of an odd C_in starts one channel early)
    const int last_first = L.C_in - 2;
    typedef std::conditional_t<WM == 2, u32x2, uint32_t> Staged;
    auto load_stage = [&](int c) -> Staged {
        const uint32_t cof = (uint32_t)min(2 * c, last_first) * plane_bytes;
        if constexpr (WM == 2) return __builtin_amdgcn_raw_buffer_load_b64(xres, (int)goff, (int)cof, 0);
        else return __builtin_amdgcn_raw_buffer_load_b32(xres, (int)goff, (int)cof, 0);
    };
    constexpr int SRING = 4;
    Staged stg[SRING];
    // the staged words of the first steps are requested as soon as the tile's first row is known
    if constexpr (STG) {
#pragma unroll
        for (int u = 0; u < SRING; ++u) stg[u] = load_stage(min(u, last));
    }
    if constexpr (STG) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        int n, ho, wo;
        const bool ok = pixel_of(pb, n_l, n, ho, wo);
        yoff[pb] = ok ? (uint32_t)((n * L.C_out + 4 * h) * L.HoWo + ho * L.Wo + wo) * 4u : 0xffffffffu;
        ptype[pb] = border_type(ho, wo, L.H, L.W, L.stride);
        const int hc = ho * L.stride, first = wo * L.stride - 1;
        const int col = first < 0 ? 0 : first;     // column of the first bit cut out
        const int jlo = WM == 1 ? 0 : col >> 5;
        const int piece = WM == 2 ? (col < 30 ? 0 : col < 46 ? 1 : 2) : 0;          // staged piece that holds columns col .. col + 2
        sh[pb] = STG ? (uint32_t)(col - 16 * piece) : (uint32_t)(col & 31);
        // the window is (bits cut out) << lsh, masked to the taps inside the image; the shift rides on the
        // multiplication by the table's row size, the mask moves in front of it
        const uint32_t lsh = (first < 0 ? 1u : 0u) + (hc == 0 ? 3u : 0u);
        wd[pb] = first < 0 ? 2u : 3u;
        wmul[pb] = 4u + lsh;                       // 16-byte part of the row: window << 4
        vm[pb] = (~border_invalid_window(ptype[pb]) & 0x1ffu) >> lsh;
        xoff[pb] = (uint32_t)(((n * L.C_in + h) * L.H + (hc == 0 ? 0 : hc - 1)) * L.WW + jlo) * 4u;
        loff[pb] = stage_wave + (uint32_t)(h * MF_STAGE_SLOTS + (n * L.H + (hc == 0 ? 0 : hc - 1) - R_first) * SW + piece) * 4u;
    }

    constexpr bool ONE_WORD = WM == 1 || STG;      // a lane cuts its window row out of one 32-bit piece
    struct Raw {
        uint32_t lo[PB][3], hi[ONE_WORD ? 1 : PB][3];
    };
    const uint32_t row_bytes = (uint32_t)L.WW * 4u;
    auto load_raw = [&](int c, Raw &r) {
        const uint32_t cof = (uint32_t)min(2 * c, last_first) * plane_bytes;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            if constexpr (WM == 1) {                 // rows are consecutive words
                const u32x3 v = __builtin_amdgcn_raw_buffer_load_b96(xres, (int)xoff[pb], (int)cof, 0);
                r.lo[pb][0] = v.x;
                r.lo[pb][1] = v.y;
                r.lo[pb][2] = v.z;
            } else if constexpr (WM == 2) {          // rows are consecutive word pairs
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(xres, (int)xoff[pb], (int)cof, 0);
                const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(xres, (int)(xoff[pb] + 16u), (int)cof, 0);
                r.lo[pb][0] = v.x;
                r.hi[pb][0] = v.y;
                r.lo[pb][1] = v.z;
                r.hi[pb][1] = v.w;
                r.lo[pb][2] = w.x;
                r.hi[pb][2] = w.y;
            } else {
#pragma unroll
                for (int dy = 0; dy < 3; ++dy) {
                    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(xres, (int)(xoff[pb] + (uint32_t)dy * row_bytes), (int)cof, 0);
                    r.lo[pb][dy] = v.x;
                    r.hi[pb][dy] = v.y;
                }
            }
        }
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
    // LDS address of the table row of pixel block pb's window (24 bytes: 32 FP6 values), and the row -> B operand
    auto row_addr = [&](const Raw &r, int pb) -> uint32_t {
        uint32_t row[3];
#pragma unroll
        for (int dy = 0; dy < 3; ++dy) {
            if constexpr (ONE_WORD) row[dy] = __builtin_amdgcn_ubfe(r.lo[pb][dy], sh[pb], wd[pb]);
            else row[dy] = __builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(r.hi[pb][dy], r.lo[pb][dy], sh[pb]), 0u, wd[pb]);
        }
        const uint32_t w = (row[0] | (row[1] << 3) | (row[2] << 6)) & vm[pb];
        return w << wmul[pb];                      // 16 x window (the shift by lsh rides along)
    };
    auto read_B = [&](uint32_t w16) -> v8i {
        const u32x4 q0 = *(lds_cu32x4 *)(uintptr_t)(lds0 + w16);
        const u32x2 q1 = *(lds_cu32x2 *)(uintptr_t)(lds0 + ST_LUT8_OFF + (w16 >> 1));
        return (v8i){(int)q0.x, (int)q0.y, (int)q0.z, (int)q0.w, (int)q1.x, (int)q1.y, 0, 0};
    };
    // one-hot rows of the CB channel blocks -> A operands (FP4 1.0 = 0b0010 in the selected nibble)
    auto make_A = [&](const uint32_t (&s)[CB], v8i (&A)[CB]) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const uint32_t sa = s[cb];
            A[cb] = (v8i){(int)__builtin_amdgcn_perm(0u, 0x00002002u, sa), (int)__builtin_amdgcn_perm(0u, 0x20020000u, sa),
                          (int)__builtin_amdgcn_perm(0x00002002u, 0u, sa), (int)__builtin_amdgcn_perm(0x20020000u, 0u, sa),
                          0, 0, 0, 0};
        }
    };

    v16f acc[CB][PB];

    const int c_end = L.npairs;

    // Pipeline.  Memory loads run RING steps ahead (a ring of RING register sets; with staging one staged
    // word per step in a ring of SRING, and the rows come out of LDS one step ahead).  The one-hot operands
    // of the next step are made during the current one (two sets).  The table rows are NOT double
    // buffered: pixel block pb's row for the next step is read into the registers of the current one as
    // soon as the block's last matrix instruction of this step has been issued, and has a whole step to
    // arrive.  A step is cut into slots by scheduling fences (nothing moves across one): each slot starts
    // with the matrix instructions of one pixel block (or half of them) and carries its share of the
    // address arithmetic, LDS traffic and loads, which run while the matrix pipe works.
    constexpr int UNROLL = STG ? SRING : RING % 2 == 0 ? RING : 2 * RING;
    static_assert(UNROLL % RING == 0 && UNROLL % 2 == 0 && (!STG || UNROLL % SRING == 0), "register sets rotate with the unrolled steps");
    Raw raw[STG ? 1 : RING];
    v8i A[2][CB], B[PB];
#pragma unroll
    for (int u = 0; u < RING; ++u) {
        if constexpr (!STG) load_raw(min(u, last), raw[u]);
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- the tables requested at the start -> LDS (only this wave reads them)
    if (new_layer) {
#pragma unroll
        for (int i = 0; i < 12; ++i) *(lds_u32x4 *)(uintptr_t)(lds0 + (uint32_t)(i * 64 + lane) * 16u) = lut_t[i];
    }
    if (lane < NCH / 4) *(lds_u32x4 *)(uintptr_t)(lds0 + ST_ALPHA_OFF + (uint32_t)lane * 16u) = tab_a;
#pragma unroll
    for (int q = 0; q < CROUNDS; ++q) {
        const int e = q * 64 + lane, type = e / CR, pc = e - type * CR;
        *(lds_u32x4 *)(uintptr_t)(lds0 + ST_CORR_OFF + (uint32_t)(type * NCH + pc * 8) * 2u) = tab_c[q];
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (STG) restage(stg[0], raw[0]);
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) B[pb] = read_B(row_addr(raw[0], pb));
    make_A(sel[0], A[0]);
    if constexpr (STG) restage(stg[1 % SRING], raw[0]);
    __builtin_amdgcn_sched_barrier(0);
    // (in the first step of a tile the sums start from a zero operand instead of 128 registers set to zero)
    auto mfma_block = [&](auto first_c, int cur, int pb, int cb_from, int cb_to) {
        constexpr bool FIRST = decltype(first_c)::value;
        const v16f zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int cb = cb_from; cb < cb_to; ++cb)
            // (scale operands of zero: the compiler then selects the instruction form without block scales, one
            // instruction word pair less to issue per matrix instruction than the scaled form with scales of 1.0)
            acc[cb][pb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A[cur][cb], B[pb], FIRST ? zero : acc[cb][pb], 4 /* A: FP4 */, 2 /* B: FP6 e2m3 */,
                                                                          0, 0, 0, 0);
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    // u = c % UNROLL selects the register sets
    auto step = [&](int c, auto uc, auto first_c) {
        constexpr int u = decltype(uc)::value;
        constexpr int cur = u % 2, nxt = (u + 1) % 2;
        constexpr int slot_next = (u + 1) % RING, slot_load = u % RING;
        uint32_t addr[PB];
        if constexpr (STG) {
            static_assert(!STG || (PB == 4 && CB == 2), "slots of the staged form");
            // slot 0: block 0; three row addresses of the next step
            mfma_block(first_c, cur, 0, 0, 2);
            addr[0] = row_addr(raw[0], 0);
            B[0] = read_B(addr[0]);
            addr[1] = row_addr(raw[0], 1);
            addr[2] = row_addr(raw[0], 2);
            fence();
            // slot 1: block 1; the last address; then the rows of step c + 2 replace those of step c + 1
            mfma_block(first_c, cur, 1, 0, 2);
            B[1] = read_B(addr[1]);
            addr[3] = row_addr(raw[0], 3);
            restage(stg[(u + 2) % SRING], raw[0]);
            fence();
            // slot 2: block 2; the one-hot operands of the next step
            mfma_block(first_c, cur, 2, 0, 2);
            B[2] = read_B(addr[2]);
            make_A(sel[slot_next], A[nxt]);
            fence();
            // slot 3: block 3; the loads of later steps
            mfma_block(first_c, cur, 3, 0, 2);
            B[3] = read_B(addr[3]);
            stg[u % SRING] = load_stage(min(c + SRING, last));
            load_sel(min(c + RING, last), sel[slot_load]);
            fence();
        } else {
            static_assert(STG || CB == 2 || (PB == 2 && CB == 4), "slots of the plain forms");
            if constexpr (CB == 4) {
                // slot 0: first half of block 0; the loads of later steps, the row addresses of the next step
                mfma_block(first_c, cur, 0, 0, 2);
                load_raw(min(c + RING, last), raw[slot_load]);
                load_sel(min(c + RING, last), sel[slot_load]);
                addr[0] = row_addr(raw[slot_next], 0);
                fence();
                // slot 1: second half of block 0, then its next row
                mfma_block(first_c, cur, 0, 2, 4);
                B[0] = read_B(addr[0]);
                addr[1] = row_addr(raw[slot_next], 1);
                fence();
                // slots 2 and 3: block 1; the one-hot operands of the next step
                mfma_block(first_c, cur, 1, 0, 2);
                make_A(sel[slot_next], A[nxt]);
                fence();
                mfma_block(first_c, cur, 1, 2, 4);
                B[1] = read_B(addr[1]);
                fence();
            } else {
                // four pixel blocks of two channel blocks, rows loaded directly (short rows that cannot be staged)
                mfma_block(first_c, cur, 0, 0, 2);
                load_raw(min(c + RING, last), raw[slot_load]);
                load_sel(min(c + RING, last), sel[slot_load]);
                addr[0] = row_addr(raw[slot_next], 0);
                B[0] = read_B(addr[0]);
                addr[1] = row_addr(raw[slot_next], 1);
                fence();
                mfma_block(first_c, cur, 1, 0, 2);
                B[1] = read_B(addr[1]);
                addr[2] = row_addr(raw[slot_next], 2);
                addr[3] = row_addr(raw[slot_next], 3);
                fence();
                mfma_block(first_c, cur, 2, 0, 2);
                B[2] = read_B(addr[2]);
                make_A(sel[slot_next], A[nxt]);
                fence();
                mfma_block(first_c, cur, 3, 0, 2);
                B[3] = read_B(addr[3]);
                fence();
            }
        }
    };
    auto group = [&](int c, auto guarded, auto first_group) {
        // UNROLL consecutive steps; the guarded form (the tail) stops at c_end
        auto run = [&](auto uc) {
            constexpr int u = decltype(uc)::value;
            if (!decltype(guarded)::value || c + u < c_end) step(c + u, uc, std::integral_constant<bool, decltype(first_group)::value && u == 0>{});
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
        if constexpr (UNROLL > 6) {
            run(std::integral_constant<int, 6>{});
            run(std::integral_constant<int, 7>{});
        }
    };
    int c = 0;
    if (UNROLL <= c_end) {
        group(0, std::false_type{}, std::true_type{});
        c = UNROLL;
    } else {                                       // fewer steps than one unrolled group: the guarded form adds to zeros
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;
    }
    for (; c + UNROLL <= c_end; c += UNROLL) group(c, std::false_type{}, std::false_type{});
    if (c < c_end) group(c, std::true_type{}, std::false_type{});
    // The worker's next item is drawn here: the counter's old value arrives while the outputs are finished.
    // (An instruction written out by hand: the compiler's own form waits for the value right away.  It is
    // looked at after an explicit wait at the end of the item; an instruction the compiler does not know
    // to be outstanding only makes its own waits longer.  Drawing earlier, at the start of the loop, was
    // measured and loses: the workers' first tiles start together, their additions to the same few words take
    // microseconds, and every load of the loop queues behind the addition it follows.)
    if (threadIdx.x == 0) asm volatile("global_atomic_add %0, %1, %2, off sc0" : "+v"(drawn) : "v"(sched), "v"(1u) : "memory");

    // ---- finishing: S = 2 M + negcorr[type][channel], y = float(S) * alpha[channel] -------------------
    // Register r of a block: output channel 8 (r / 4) + 4 h + r % 4, pixel n_l.  The lane reads alpha
    // and the correction of its four consecutive channels with one access each; the fused
    // multiply-add is exact (integers below 2^24), so y is the one rounding of float(S) * alpha.
    int lane_f = threadIdx.x;
    asm volatile("" : "+v"(lane_f));
    const int h_f = lane_f >> 5;
    const __amdgpu_buffer_rsrc_t yres = make_rsrc(L.y, (uint32_t)((size_t)L.N * L.C_out * L.HoWo * 4u));
    const uint32_t chan_bytes = (uint32_t)L.HoWo * 4u;
    auto value = [&](int cb, int pb, int r, const u32x4 (&al)[4], const u32x2 (&cr)[4]) -> float {
        const int j = r / 4, i = r % 4;
        const uint32_t pairw = i < 2 ? cr[j].x : cr[j].y;
        const int nc = (i & 1) ? (int)pairw >> 16 : (int)(pairw << 16) >> 16;
        const float a = __uint_as_float(i == 0 ? al[j].x : i == 1 ? al[j].y : i == 2 ? al[j].z : al[j].w);
        return __builtin_fmaf(acc[cb][pb][r], 2.0f, (float)nc) * a;
    };
    // One 4-byte non-temporal store per output: the 32 lanes of a half write 128 contiguous bytes of one channel
    // plane.  (Measured against 16-byte stores of four pixels after a transposition of half blocks through LDS: that
    // form needs a quarter of the store instructions but pays eight LDS writes and two reads per half block, and the
    // launch is 1.5 % slower with it.)
    const int ch_left = L.C_out - co0 - 4 * h_f;                   // channel c of the tile (lane half 0) exists if c < ch_left
    // A tile whose channels all exist (every tile unless C_out is not a multiple of the tile's channels, and then
    // only the last channel tile) skips the per-store test: a quarter of the finishing step's instructions.
    auto finish = [&](auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            u32x4 al[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) al[j] = *(lds_cu32x4 *)(uintptr_t)(lds0 + ST_ALPHA_OFF + (uint32_t)(cb * 32 + 8 * j + 4 * h_f) * 4u);
            u32x2 cr[PB][4];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    cr[pb][j] = *(lds_cu32x2 *)(uintptr_t)(lds0 + ST_CORR_OFF + (uint32_t)(ptype[pb] * NCH + cb * 32 + 8 * j + 4 * h_f) * 2u);
            // a channel's pixel blocks one after the other: consecutive blocks of an image are adjacent in its plane
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cs = co0 + cb * 32 + 8 * (r / 4) + r % 4;      // wave-uniform part of the channel
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    // channels past C_out (padding of the last block) are not stored: their lanes get an offset outside the tensor
                    const uint32_t at = FULL || cb * 32 + 8 * (r / 4) + r % 4 < ch_left ? yoff[pb] : 0xffffffffu;
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(value(cb, pb, r, al, cr[pb])), yres, (int)at,
                                                          (int)((uint32_t)cs * chan_bytes), 2 /* nt */);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (co0 + NCH <= L.C_out) finish(std::true_type{});
    else finish(std::false_type{});
}

__global__ __launch_bounds__(64, 2)
void subbit_stack_kernel(const StackParams sp)
{
    __shared__ __align__(16) unsigned char smem[ST_LDS_BYTES];
    // (A static array, and its address taken from a pointer in the LDS address space: the compiler then knows the
    // address as a constant and folds it into the offset fields of the LDS instructions.  The address of a
    // dynamically sized array is only fixed at link time, and through a generic pointer it is a run-time value
    // behind a null check: either way every table access paid an addition, an eighth of the loops' vector
    // instructions.)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int lane = threadIdx.x;
    int cur_layer = -1;
    // The run table sits in the wave's LDS, one run per lane, so that finding an item's run is one read
    // and one ballot instead of a chain of dependent scalar loads.
    {
        u32x2 e;
        e.x = lane < sp.n_runs ? (uint32_t)sp.run_first_item[lane] : 0x7fffffffu;
        e.y = (uint32_t)sp.run_first_tile[lane] | (uint32_t)sp.run_layer[lane] << 24;       // tiles of a layer < 2^24
        *(__attribute__((address_space(3))) u32x2 *)(uintptr_t)(lds0 + ST_RUNS_OFF + (uint32_t)lane * 8u) = e;
    }
    // Items are handed out by ST_QUEUES counters, one per XCD: queue q owns the groups q, q + ST_QUEUES, ... of
    // ST_GROUP consecutive items, and its draw number j is item ((j / ST_GROUP) * ST_QUEUES + q) * ST_GROUP +
    // j % ST_GROUP.  A worker draws from the queue of the XCD it runs on, so the tiles an XCD works on at any time
    // are neighbours in their layers - they share the cache lines of their input rows (a 128-byte line of packed
    // rows holds 16 or 32 image rows of a channel) and of the output planes' ends in that XCD's L2 instead of
    // fetching them once per XCD - while all queues still advance through the item order at the same pace.  A
    // worker whose queue is empty takes from the next queue that is not (a plain look at all counters picks it;
    // an empty draw marks a queue as finished for this worker, so the search ends after at most ST_QUEUES
    // rounds whatever the loads return), so every item is handed out whichever XCDs the workers sit on.
    // The next item is drawn while the current one's outputs are finished (see stack_tile).
    auto item_of = [](uint32_t j, uint32_t q) { return (((j >> ST_GROUP_LOG2) * ST_QUEUES + q) << ST_GROUP_LOG2) | (j & (ST_GROUP - 1u)); };
    uint32_t queue = (__builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11)) & 15u) % ST_QUEUES;      // XCC_ID
    uint32_t finished = 0;                       // queues this worker has found empty
    uint32_t drawn = 0;
    // The first draws of every queue are not drawn at all: worker b takes draw b / ST_QUEUES of queue b % ST_QUEUES
    // (workgroups go to the XCDs in turn, so this is its own queue, and if not the item is still handed out
    // once), and a counter's value c stands for draw n_static + c.  Two thousand additions at the start of a
    // launch would take longer than the set-up of a tile.
    const uint32_t n_static = (uint32_t)sp.n_workers / ST_QUEUES;
    uint32_t item;
    if (blockIdx.x < n_static * ST_QUEUES) {
        item = item_of(blockIdx.x / ST_QUEUES, blockIdx.x % ST_QUEUES);
    } else {
        if (lane == 0) drawn = atomicAdd(sp.sched + queue * MF_SCHED_STRIDE, 1u);
        item = item_of(n_static + (uint32_t)__builtin_amdgcn_readfirstlane((int)drawn), queue);
    }
    for (;;) {
        while (item >= (uint32_t)sp.n_items) {
            finished |= 1u << queue;
            uint32_t c = 0xffffffffu - n_static;
            if (lane < (int)ST_QUEUES) c = __hip_atomic_load(sp.sched + lane * MF_SCHED_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool has = lane < (int)ST_QUEUES && item_of(n_static + c, (uint32_t)lane) < (uint32_t)sp.n_items;
            const uint32_t open = (uint32_t)__ballot(has) & ~finished;
            if (open == 0u) break;
            // the first open queue after this one, cyclically
            const uint32_t rot = ((open >> queue) | (open << (ST_QUEUES - queue))) & ((1u << ST_QUEUES) - 1u);
            queue = (queue + (uint32_t)__builtin_ctz(rot)) % ST_QUEUES;
            if (lane == 0) drawn = atomicAdd(sp.sched + queue * MF_SCHED_STRIDE, 1u);
            item = item_of(n_static + (uint32_t)__builtin_amdgcn_readfirstlane((int)drawn), queue);
        }
        if (item >= (uint32_t)sp.n_items) break;
        uint32_t *const counter = sp.sched + queue * MF_SCHED_STRIDE;
        // Position in the run table.  The table lists the tiles bound by the matrix pipe first, then those bound
        // by LDS; the items deal from both lists in proportion, so that at any time a compute unit holds waves
        // of both kinds: with j(i) = mulhi(i, deal_ratio) - monotone, steps of at most one, j(n_items) = size
        // of the second list - item i is entry j(i) of the second list where j steps up, else entry i - j(i)
        // of the first.
        // The end of the queue is not dealt: it is the end of the first list alone, whose short tiles run faster
        // the fewer waves are left, so that the launch does not end on LDS-bound tiles.
        uint32_t pos = item;
        const uint32_t n_head = (uint32_t)(sp.n_items - sp.n_tail);
        if (item >= n_head) {
            pos = (uint32_t)(sp.n_matrix_items - sp.n_tail) + (item - n_head);
        } else if (sp.deal_ratio != 0u) {
            const uint32_t j0 = __umulhi(item, sp.deal_ratio), j1 = __umulhi(item + 1u, sp.deal_ratio);
            pos = j1 > j0 ? (uint32_t)sp.n_matrix_items + j0 : item - j0;
        }
        const u32x2 run = *(lds_cu32x2 *)(uintptr_t)(lds0 + ST_RUNS_OFF + (uint32_t)lane * 8u);
        const int r = __builtin_popcountll(__ballot((int)pos >= (int)run.x)) - 1;      // the last run that starts at or before it
        const uint32_t rt = (uint32_t)__builtin_amdgcn_readlane((int)run.y, r);
        const int l = (int)(rt >> 24);
        const int tile = (int)(rt & 0xffffffu) + ((int)pos - __builtin_amdgcn_readlane((int)run.x, r));
        const StackLayer &L = sp.layer[l];
        const bool new_layer = l != cur_layer;
        cur_layer = l;
        switch (L.variant) {
        case 1: stack_tile<4, 2, 1, false>(L, tile, lds0, new_layer, counter, drawn); break;
        case 3: stack_tile<4, 2, 1, true>(L, tile, lds0, new_layer, counter, drawn); break;
        case 4: stack_tile<4, 2, 2, true>(L, tile, lds0, new_layer, counter, drawn); break;
        case 5: stack_tile<2, 4, 0, false>(L, tile, lds0, new_layer, counter, drawn); break;
        case 6: stack_tile<2, 4, 1, false>(L, tile, lds0, new_layer, counter, drawn); break;
        default: stack_tile<2, 4, 2, false>(L, tile, lds0, new_layer, counter, drawn); break;
        }
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(drawn) : : "memory");
        item = item_of(n_static + (uint32_t)__builtin_amdgcn_readfirstlane((int)drawn), queue);
    }
    // The last worker to leave puts the scheduling words back to zero for the next launch: by
    // then every other worker has drawn its last item and counted itself.
    if (lane == 0) {
        uint32_t *const leave = sp.sched + ST_QUEUES * MF_SCHED_STRIDE;
        const uint32_t left = atomicAdd(leave, 1u);
        if (left == (uint32_t)sp.n_workers - 1u) {
            for (uint32_t q = 0; q < ST_QUEUES; ++q) atomicExch(sp.sched + q * MF_SCHED_STRIDE, 0u);
            atomicExch(leave, 0u);
        }
    }
}

int stack_variant(const MfPlan &pl, const Geom &g)
{
    if (pl.one || pl.quad || !pl.pair || g.C_in > 3000) return -1;
    const int wm = g.WW <= 2 ? g.WW : 0;
    // (tiles of four pixel blocks whose rows are two or more words and cannot be staged would need more
    // registers than two waves per SIMD leave: such layers go through the per-layer kernel)
    if (pl.cfg.PB == 4 && pl.cfg.CB == 2) return pl.stage ? (wm == 1 ? 3 : 4) : wm == 1 ? 1 : -1;
    if (pl.cfg.PB == 2 && pl.cfg.CB == 4 && !pl.stage) return 5 + wm;
    return -1;
}

int device_compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        cus = n;
    }
    return cus;
}

}  // namespace

bool subbit_stack_supported(int n_layers, const Geom *gs)
{
    if (n_layers < 1 || n_layers > ST_MAX_LAYERS) return false;
    for (int l = 0; l < n_layers; ++l) {
        if (!subbit_mfma_supported(gs[l])) return false;
        const MfPlan pl = mf_plan(gs[l]);
        if (stack_variant(pl, gs[l]) < 0 || pl.n_tiles > 0xffffffLL || pl.n_pxblocks > 0x7fffffffLL) return false;
    }
    return true;
}

// Layers: prepared workspaces (fp32 form), each with its own input and output.
int launch_subbit_stack(int n_layers, const Geom *gs, const void *const *x, float *const *y, void *const *ws, hipStream_t s)
{
    StackParams sp;
    struct Item {
        int layer;
        long long tiles;
        long long weight;     // matrix instructions per tile
        bool lds_bound;       // two channel blocks per wave
    };
    std::vector<Item> order;
    long long total = 0;
    for (int l = 0; l < n_layers; ++l) {
        const Geom &g = gs[l];
        const MfPlan pl = mf_plan(g);
        StackLayer &L = sp.layer[l];
        L.x = (const uint32_t *)x[l];
        L.lut = (const uint32_t *)((char *)ws[l] + pl.off_lut);
        L.sel = (const uint32_t *)((char *)ws[l] + pl.off_sel);
        L.negcorr = (const int16_t *)((char *)ws[l] + pl.off_negcorr);
        L.alpha = (const float *)((char *)ws[l] + pl.off_alphap);
        L.y = y[l];
        L.N = g.N; L.C_in = g.C_in; L.C_out = g.C_out; L.H = g.H; L.W = g.W; L.stride = g.stride;
        L.Ho = g.Ho; L.Wo = g.Wo; L.HoWo = g.HoWo; L.WW = g.WW; L.P = (int)g.P;
        L.COP = pl.COP; L.npairs = pl.npairs; L.n_cotiles = pl.n_cotiles; L.n_pxblocks = (int)pl.n_pxblocks;
        L.variant = stack_variant(pl, g);
        L.div_HoWo = make_divisor((uint32_t)g.HoWo);
        L.div_Wo = make_divisor((uint32_t)g.Wo);
        L.div_H = make_divisor((uint32_t)g.H);
        L.div_cotiles = make_divisor((uint32_t)pl.n_cotiles);
        if (L.variant < 0) return SNN_ERR_UNSUPPORTED;
        order.push_back({l, pl.n_tiles, (long long)pl.npairs * pl.cfg.PB * pl.cfg.CB, pl.cfg.CB == 2});
        total += pl.n_tiles;
    }
    if (total > 0x7fffffffLL) return SNN_ERR_UNSUPPORTED;
    // Order of the items: two lists, each longest tile first - the layers whose tiles are bound by the matrix
    // pipe (four channel blocks per wave: one table row feeds four matrix instructions) and those bound by LDS
    // (two channel blocks: a row per two instructions, plus the staged input rows).  The kernel deals items from
    // both in proportion, so that waves of both kinds share every compute unit for the whole launch instead of
    // the LDS-bound layers running by themselves at the end.  The queue is dynamic; the last items are the
    // shortest of their lists.
    std::stable_sort(order.begin(), order.end(), [](const Item &a, const Item &b) {
        if (a.lds_bound != b.lds_bound) return !a.lds_bound;
        return a.weight > b.weight;
    });
    const long long want = (long long)device_compute_units() * ST_WORKERS_PER_CU;
    const long long n_workers = std::min<long long>(want, total);
    struct Run {
        int layer;
        long long t0, n;
    };
    std::vector<Run> runs;
    long long n_matrix = 0;
    for (const Item &it : order) {
        runs.push_back({it.layer, 0, it.tiles});
        if (!it.lds_bound) n_matrix += it.tiles;
    }
    sp.n_matrix_items = (int)n_matrix;
    // the last items: one per worker from the end of the matrix-bound list (its shortest tiles), where both lists exist
    // (measured: 2 % of the launch; half or one and a half times as many make no difference, more loses)
    const long long n_tail = n_matrix == total || n_matrix <= n_workers ? 0 : n_workers;
    const long long dealt = total - n_tail;
    sp.n_tail = (int)n_tail;
    sp.deal_ratio = n_matrix == 0 || n_matrix == total ? 0u : (uint32_t)((((unsigned long long)(total - n_matrix) << 32) + dealt - 1) / dealt);
    if ((int)runs.size() > ST_MAX_RUNS) return SNN_ERR_UNSUPPORTED;
    int n_runs = 0;
    long long first = 0;
    for (const Run &r : runs) {
        sp.run_first_item[n_runs] = (int)first;
        sp.run_first_tile[n_runs] = (int)r.t0;
        sp.run_layer[n_runs] = (unsigned char)r.layer;
        first += r.n;
        ++n_runs;
    }
    for (int r = n_runs; r <= ST_MAX_RUNS; ++r) sp.run_first_item[r] = (int)first;
    for (int r = n_runs; r < ST_MAX_RUNS; ++r) {
        sp.run_first_tile[r] = 0;
        sp.run_layer[r] = 0;
    }
    sp.n_runs = n_runs;
    sp.n_items = (int)total;
    sp.n_workers = (int)n_workers;
    sp.sched = (uint32_t *)((char *)ws[0] + mf_plan(gs[0]).off_sched);
    hipLaunchKernelGGL(subbit_stack_kernel, dim3((unsigned)sp.n_workers), dim3(64), 0, s, sp);
    return check_launch();
}

}  // namespace snn
