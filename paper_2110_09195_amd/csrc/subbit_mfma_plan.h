// Plan of the matrix-core sub-bit convolution (host side): tile shape, channel split, table layout in
// the workspace.  Shared by the translation units that launch kernels on those tables.
#pragma once

#include "snn_internal.h"

namespace snn {

constexpr int MF_WAVES = 4;                    // waves per workgroup
constexpr int MF_STAGE_SLOTS = 32;             // packed words a wave stages per input channel and step
// scheduling words of the launch that walks a stack: one item counter per queue, 128 bytes apart (a queue per XCD:
// its own cache line), then the count of workers that have left
constexpr int MF_SCHED_QUEUES = 8;
constexpr int MF_SCHED_STRIDE = 32;
constexpr int MF_SCHED_WORDS = MF_SCHED_QUEUES * MF_SCHED_STRIDE + 1;
constexpr int MF_STAGE_BYTES = 2 * MF_STAGE_SLOTS * 4 + 32;   // per wave: two channels + room for reads past the last slot
// Table row stride in LDS: 24 bytes (32 FP6 values) per lane half, each half padded to 32 bytes in
// the two-half form, the row padded to an odd number of 16-byte pieces (fewer bank conflicts).
__host__ __device__ constexpr int mf_lrow(bool pair) { return pair ? 48 : 80; }

// Two-channel form (subsets of up to 32 members): the table image is 512 rows of 6 words; a second image in
// "split" order (words 0-3 of every row, then words 4-5 of every row) follows it MF_LUT_SPLIT_WORDS words in.
constexpr int MF_LUT_SPLIT_WORDS = 512 * 6;

struct MfCfg {
    int PB, CB;
};

struct MfPlan {
    MfCfg cfg;
    bool pair;        // K <= 32: two input channels per step
    bool quad;        // K <= 16 (3x3 layers): four
    bool stage;       // the rows of a tile fit the staging slots
    bool one;         // 1x1 layer (g.C_in = groups of 8 input channels)
    int KS, COP, n_cotiles, npairs;
    long long n_pxblocks, n_pxtiles, n_tiles, n_wgs;
    size_t lds;
    size_t off_sel, off_fin, off_lut, bytes;
    // read by the launch that walks a stack of layers with one resident wave per work slot (fp32 output only):
    size_t off_negcorr;   // int16 [16][COP]: minus the finishing table's correction term, border type major
    size_t off_alphap;    // float [COP]: alpha padded with zeros
    size_t off_sched;     // MF_SCHED_WORDS scheduling words of the stack launch; zero between launches
};

// blocks of up to 32 pixels: 32 consecutive pixels each, or (sign epilogue) whole output words
inline int64_t mf_pxblocks(const Geom &g, bool aligned)
{
    if (!aligned) return (g.P + 31) / 32;
    if (g.Wo <= 32) {
        const int rows_pb = 32 / g.Wo;
        return (int64_t)g.N * ((g.Ho + rows_pb - 1) / rows_pb);
    }
    return (int64_t)g.N * g.Ho * ((g.Wo + 31) / 32);
}

inline MfPlan mf_plan(const Geom &g, bool aligned = false, bool one = false)
{
    MfPlan pl;
    pl.one = one;
    // tile of a wave: 128 accumulator registers (PB x CB = 8); few channels -> more pixels per wave
    if (g.C_out <= 64) pl.cfg = {4, 2};
    else pl.cfg = {2, 4};
    if (const int t = tuning(SNN_TUNE_MFMA_TILE); t > 0) pl.cfg = {t / 10, t % 10};
    const int cow = 32 * pl.cfg.CB, pxw = 32 * pl.cfg.PB;
    pl.COP = (g.C_out + cow - 1) / cow * cow;
    pl.n_cotiles = pl.COP / cow;
    pl.n_pxblocks = mf_pxblocks(g, aligned);
    pl.n_pxtiles = (pl.n_pxblocks + pl.cfg.PB - 1) / pl.cfg.PB;
    pl.n_tiles = pl.n_pxtiles * pl.n_cotiles;
    pl.pair = g.K <= 32;
    pl.quad = false;
    pl.npairs = pl.pair ? (g.C_in + 1) / 2 : g.C_in;
    // split the channel pairs over waves while the tiles alone leave SIMDs idle (1024 SIMDs, two waves each)
    auto split_of = [&](int steps) {
        int ks = 1;
        while (ks < 4 && pl.n_tiles * ks < 1536 && steps / (2 * ks) >= 8) ks *= 2;
        return ks;
    };
    int KS = split_of(pl.npairs);
    // Subsets of at most 16 members: four channels per step halve the matrix instructions and double the
    // window work of a step (and give up the staged rows).  Measured: a gain (1.2x) only where a wave has
    // long runs of steps - many input channels on tiles of four channel blocks - and a loss on short ones.
    // The knob SNN_TUNE_MFMA_QUAD = 1 / 0 forces it on wherever it applies / off.
    if (g.K <= 16 && !one) {
        const int quad_env = tuning(SNN_TUNE_MFMA_QUAD);
        const bool pays = pl.cfg.CB == 4 && (int64_t)(pl.npairs / KS) * pl.cfg.PB * pl.cfg.CB >= 768;
        if (quad_env < 0 ? pays : quad_env != 0) {
            pl.quad = true;
            pl.npairs = (g.C_in + 3) / 4;
            KS = split_of(pl.npairs);
        }
    }
    if (const int ks = tuning(SNN_TUNE_MFMA_KS); ks > 0) KS = ks;
    pl.KS = KS;
    pl.n_wgs = (pl.n_tiles * KS + MF_WAVES - 1) / MF_WAVES;
    // Rows a tile of pxw consecutive pixels can touch, numbered over the whole batch: a change of
    // output row moves the first row loaded by at most `stride`, a change of image by one more
    // (the top row of an image is not preceded by a padding row), and the last pixel loads three.
    const int64_t row_changes = (g.Wo - 1 + pxw - 1) / g.Wo, image_changes = ((int64_t)g.HoWo - 1 + pxw - 1) / g.HoWo;
    const int64_t tile_rows = g.stride * row_changes + image_changes + 3;
    // Staging pays where the memory pipeline is the bound: two channel blocks per wave, i.e. only two
    // matrix instructions per window (measured; with four blocks the loop is bound by the matrix pipe
    // and the extra LDS traffic costs a little).  The knob SNN_TUNE_MFMA_STAGE = 1 / 0 forces it on wherever it fits / off.
    const int stage_env = tuning(SNN_TUNE_MFMA_STAGE);
    pl.stage = !one && !pl.quad && g.WW <= 2 && tile_rows * (g.WW == 2 ? 3 : 1) <= MF_STAGE_SLOTS &&
               (stage_env < 0 ? pl.cfg.CB == 2 : stage_env != 0);
    const size_t lut_bytes = (size_t)(one ? 256 : 512) * mf_lrow(pl.pair) + (pl.stage ? (size_t)MF_WAVES * MF_STAGE_BYTES : 0);
    const int nblk = pl.cfg.PB * pl.cfg.CB;
    const size_t red_bytes = KS > 1 ? (size_t)(MF_WAVES / KS) * (nblk > 4 ? nblk / 2 : nblk) * (KS - 1) * 4096 : 0;
    const size_t fin_bytes = (size_t)MF_WAVES * 32 * pl.cfg.CB * 16 * 8;
    pl.lds = lut_bytes > red_bytes ? lut_bytes : red_bytes;
    if (fin_bytes > pl.lds) pl.lds = fin_bytes;
    size_t o = 0;
    pl.off_sel = o;
    o += align_up((size_t)pl.npairs * (pl.quad ? 4 : 2) * pl.COP * sizeof(uint32_t), 256);
    pl.off_fin = o;
    o += align_up((size_t)pl.COP * 16 * sizeof(uint2), 256);
    pl.off_lut = o;
    o += align_up((size_t)512 * mf_lrow(pl.pair), 256);
    pl.off_negcorr = o;
    o += align_up((size_t)16 * pl.COP * sizeof(int16_t), 256);
    pl.off_alphap = o;
    o += align_up((size_t)pl.COP * sizeof(float), 256);
    pl.off_sched = o;
    o += align_up((size_t)MF_SCHED_WORDS * sizeof(uint32_t), 256);
    pl.bytes = o;
    return pl;
}

}  // namespace snn
