// mp8_gemm_fp8: the FP8 compute primitive of Section 3 (arXiv 1905.12334) for gfx950 --
// two 8-bit (1,5,2) operands, FP32 accumulation on the matrix cores, and the Q node of
// Figure 1a (one rounding of the complete FP32 sum to 8 bits, RNE or stochastic) fused into
// the epilogue.  The three training GEMMs (forward, backward-data, weight-gradient) are the
// same contraction  out[r,c] = sum_j a[r,j] * b[c,j]  on differently oriented operands.
//
// This file is the host side: kernel table, choice of kernel and contraction slices, argument
// checks and launches.  The kernels live in headers of their own:
//   gemm_common.hpp   argument structs, the epilogue of a run of outputs, direct-to-LDS loads
//   gemm_mfma.hpp     the general kernel: block tile BM x BN, ring of 2-4 stages of 128 bytes of
//                     contraction, slot-scheduled MFMA loop, every operand layout, 3x3 convolutions
//   gemm_shortk.hpp   contractions of one or two stages (all start-up and epilogue)
//   gemm_wavek.hpp    small outputs with long contractions (contraction divided among waves)
//   gemm_wave128.hpp  about one 128x128 tile per CU and a long contraction (every wave the whole tile)
//   gemm_finish.hpp   second pass for split contractions and unfused epilogues, optionally with
//                     the master-weight update; the any-shape fallback kernel
// Split contraction, FP32 / transposed outputs, ragged column counts: the MFMA kernels write
// FP32 tiles and the second pass sums the slices in order and applies the epilogue -- the sum
// is rounded exactly once.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "../../include/mp8.h"
#include "gemm_common.hpp"
#include "gemm_finish.hpp"
#include "gemm_mfma.hpp"
#include "gemm_shortk.hpp"
#include "gemm_wavek.hpp"
#include "gemm_wave128.hpp"
#include "gemm_qfwd.hpp"

namespace mp8 {

// ---------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------
struct TileConfig {
    int bm, bn;
    const char *name;
    void (*kernel[3])(const GemmArgs);     // indexed by EPI_*
    void (*kernel_tn[3])(const GemmArgs);  // both operands contraction-major; null if not built
    void (*kernel_bt[3])(const GemmArgs);  // only b contraction-major; null if not built
    void (*kernel_conv[3][3])(const GemmArgs);  // [mp8_op][EPI_*] 3x3 convolution; null if not built
    int max_ksteps;      // 0: any contraction length; else the most stages the kernel takes
    int lds_per_stage;   // dynamic LDS bytes per stage (kernels that load all stages at once)
};

#define MP8_TILE(BM, BN, WGM, WGN, NS, MB)                                   \
    {BM, BN, #BM "x" #BN "x128s" #NS,                                         \
     {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL>,                \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE>,                    \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL>},                  \
     {nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr},                \
     {{nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}}, 0, 0}
#define MP8_TILE_TN(BM, BN, WGM, WGN, NS, MB)                                \
    {BM, BN, #BM "x" #BN "x128s" #NS,                                         \
     {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL>,                \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE>,                    \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL>},                  \
     {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL, true, true>,    \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE, true, true>,        \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL, true, true>},      \
     {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL, false, true>,   \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE, false, true>,       \
      gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL, false, true>},      \
     {{gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL, false, true, 1>, \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE, false, true, 1>,     \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL, false, true, 1>},   \
      {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL, false, false, 2>, \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE, false, false, 2>,    \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL, false, false, 2>},  \
      {gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_PARTIAL, true, true, 3>,  \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_RNE, true, true, 3>,      \
       gemm_mfma_kernel<BM, BN, WGM, WGN, NS, MB, EPI_FULL, true, true, 3>}}, 0, 0}
#define MP8_TILE_SHORTK                                                      \
    {128, 128, "128x128x128k",                                                \
     {gemm_shortk_kernel<EPI_PARTIAL>, gemm_shortk_kernel<EPI_RNE>, gemm_shortk_kernel<EPI_FULL>}, \
     {nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr},                \
     {{nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}}, 2, 32768}
#define MP8_WAVEK(ATN, BTN, CONV)                                            \
    {gemm_wavek_kernel<EPI_PARTIAL, ATN, BTN, CONV>, gemm_wavek_kernel<EPI_RNE, ATN, BTN, CONV>, \
     gemm_wavek_kernel<EPI_FULL, ATN, BTN, CONV>}
#define MP8_TILE_WAVEK                                                       \
    {64, 64, "64x64x128w", MP8_WAVEK(false, false, 0), MP8_WAVEK(true, true, 0),  \
     MP8_WAVEK(false, true, 0),                                                \
     {{nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}, MP8_WAVEK(true, true, 3)}, 0, 0}
#define MP8_WAVEK32(BTN, BN)                                                 \
    {gemm_wavek_kernel<EPI_PARTIAL, false, BTN, 0, 32, BN>, gemm_wavek_kernel<EPI_RNE, false, BTN, 0, 32, BN>, \
     gemm_wavek_kernel<EPI_FULL, false, BTN, 0, 32, BN>}
#define MP8_NO_KERNELS {nullptr, nullptr, nullptr}
#define MP8_WAVE128(ATN, BTN)                                                \
    {gemm_wave128_kernel<EPI_PARTIAL, ATN, BTN>, gemm_wave128_kernel<EPI_RNE, ATN, BTN>, \
     gemm_wave128_kernel<EPI_FULL, ATN, BTN>}
#define MP8_TILE_WAVE128                                                     \
    {128, 128, "128x128x128p", MP8_WAVE128(false, false), MP8_WAVE128(true, true), MP8_WAVE128(false, true), \
     {MP8_NO_KERNELS, MP8_NO_KERNELS, MP8_NO_KERNELS}, 0, 0}
#define MP8_TILE_WAVEK32x64                                                  \
    {32, 64, "32x64x128w", MP8_WAVEK32(false, 64), MP8_NO_KERNELS, MP8_WAVEK32(true, 64), \
     {MP8_NO_KERNELS, MP8_NO_KERNELS, MP8_NO_KERNELS}, 0, 0}
#define MP8_TILE_WAVEK32x32                                                  \
    {32, 32, "32x32x128w", MP8_WAVEK32(false, 32), MP8_NO_KERNELS, MP8_NO_KERNELS, \
     {MP8_NO_KERNELS, MP8_NO_KERNELS, MP8_NO_KERNELS}, 0, 0}
static const TileConfig kTiles[] = {
    MP8_TILE_TN(256, 256, 2, 2, 2, 1), MP8_TILE(256, 128, 2, 2, 3, 1), MP8_TILE(128, 256, 2, 2, 3, 1),
    MP8_TILE_TN(128, 128, 2, 2, 2, 2), MP8_TILE_TN(128, 128, 2, 2, 4, 1), MP8_TILE(64, 128, 1, 4, 3, 2),
    MP8_TILE(128, 64, 4, 1, 3, 2),  MP8_TILE_TN(64, 64, 2, 2, 4, 2), MP8_TILE(64, 128, 1, 4, 2, 3),
    MP8_TILE(128, 64, 4, 1, 2, 3),  MP8_TILE_TN(64, 64, 2, 2, 2, 4),   MP8_TILE_SHORTK,
    MP8_TILE_WAVEK, MP8_TILE_WAVEK32x64, MP8_TILE_WAVEK32x32, MP8_TILE_WAVE128,
};
constexpr int kNumTiles = (int)(sizeof(kTiles) / sizeof(kTiles[0]));
constexpr int kCUs = 256;
constexpr int kMaxSplits = 64;

struct Plan {
    bool mfma;
    int tile;    // index into kTiles
    int splits;
    int tiles_m, tiles_n;
};

static void op_dims(mp8_op op, int64_t M, int64_t N, int64_t K, int64_t &rows, int64_t &cols,
                    int64_t &kc) {
    switch (op) {
        case MP8_FWD: rows = M; cols = N; kc = K; break;
        case MP8_BWD_DATA: rows = M; cols = K; kc = N; break;
        default: rows = K; cols = N; kc = M; break;
    }
}

// Choose tile shape and number of contraction slices.  Measured on MI355X: the 256x256 tile
// is the only one that approaches the matrix-core peak (fewest LDS and L2 bytes per flop) but
// needs enough tiles to fill whole rounds of 256 CUs; 128x128 serves mid-sized outputs (two
// resident blocks per CU when the contraction is short, a deeper ring when it is long); small
// outputs take 64x64 tiles and, if even those are too few, a split contraction -- kept to a
// minimum because the second pass costs several microseconds.
enum { T256x256 = 0, T128x128s2 = 3, T128x128s4 = 4, T128x64s2 = 9, T64x64s2 = 10, T128x128k = 11, T64x64w = 12,
       T32x64w = 13, T32x32w = 14, T128x128p = 15 };
static Plan make_plan(int64_t rows, int64_t cols, int64_t kc, int tile_config, int split_k,
                      int layout = 0,      // bit 0: a contraction-major, bit 1: b
                      bool conv = false) { // a convolution: only the tiles with convolution addressing
    Plan pl{};
    pl.mfma = (kc % BK) == 0 && kc > 0;
    // contraction-major operands are fetched in 16-row chunks, by the tiles built for them
    if ((layout & 1) && (rows & 15) != 0) pl.mfma = false;
    if ((layout & 2) && (cols & 15) != 0) pl.mfma = false;
    if (layout != 0 && tile_config > 0 &&
        (layout == 3 ? kTiles[tile_config - 1].kernel_tn[0] : kTiles[tile_config - 1].kernel_bt[0]) == nullptr)
        pl.mfma = false;
    const bool tn = layout != 0;
    if (layout == 0 && tile_config > 0 && kTiles[tile_config - 1].kernel[0] == nullptr) pl.mfma = false;
    if (tile_config > 0 && kTiles[tile_config - 1].max_ksteps > 0 &&
        (tn || kc / BK > kTiles[tile_config - 1].max_ksteps))
        pl.mfma = false;
    if (!pl.mfma) {
        pl.splits = 1;
        return pl;
    }
    const int ksteps = (int)(kc / BK);
    auto count = [&](int t) {
        return ((rows + kTiles[t].bm - 1) / kTiles[t].bm) * ((cols + kTiles[t].bn - 1) / kTiles[t].bn);
    };
    int t;
    if (tile_config > 0) {
        t = tile_config - 1;
    } else {
        const int64_t n256 = count(T256x256), n128 = count(T128x128s2);
        const double fill256 = (double)n256 / (double)(((n256 + kCUs - 1) / kCUs) * kCUs);
        const int64_t n64 = count(T64x64s2);
        // 128x128 tiles, one workgroup per CU, long contraction: every wave the whole tile on a
        // quarter of the contraction (measured 6-17 % faster than the four-stage ring when no CU
        // gets more than two tiles; with more tiles, or a split contraction, the ring kernels win)
        const int long128 = (!conv && n128 >= kCUs / 2 && n128 <= 2 * kCUs) ? T128x128p : T128x128s4;
        if (n256 >= 208 && fill256 >= 0.8 && ksteps >= 8) t = T256x256;
        // so few tiles that most CUs would idle and the contraction is too short to split:
        // half the rows per tile, and half the columns too if that still fits one round
        else if (layout == 0 && 4 * n64 <= kCUs && ksteps >= 16 && ksteps <= 40 && count(T32x32w) <= kCUs)
            t = T32x32w;
        else if (!(layout & 1) && 2 * n64 <= kCUs && ksteps >= 16 && ksteps <= 40 && count(T32x64w) <= kCUs)
            t = T32x64w;
        else if (n64 <= kCUs && ksteps >= 16) t = T64x64w;  // one workgroup per CU, one round
        else if (tn && (n128 < 16 || (n128 < 192 && ksteps <= 64))) t = T64x64s2;
        else if (tn) t = ksteps >= 64 ? long128 : T128x128s2;
        else if (n128 >= 192 && ksteps <= 2) t = T128x128k;  // all prologue and epilogue
        else if (n128 >= 192) t = (ksteps >= 64 && n128 <= 2 * kCUs) ? long128 : T128x128s2;
        else t = T64x64s2;
    }
    pl.tile = t;
    pl.tiles_m = (int)((rows + kTiles[t].bm - 1) / kTiles[t].bm);
    pl.tiles_n = (int)((cols + kTiles[t].bn - 1) / kTiles[t].bn);
    const int64_t nt = (int64_t)pl.tiles_m * pl.tiles_n;
    int s = 1;
    if (kTiles[t].max_ksteps > 0) {
        s = 1;  // these kernels take the whole contraction at once
    } else if (split_k == 0 && (t == T32x64w || t == T32x32w)) {
        s = 1;
    } else if (split_k == 0 && t == T64x64w) {
        // one workgroup per CU and never more workgroups than CUs (a second round would double
        // the time); at least two stages for each of the four waves.  A split costs the finishing
        // pass (about 4 us, the time of some 32 stages of one wave), so it must save more than that.
        s = (int)std::max<int64_t>(1, std::min<int64_t>(kCUs / nt, ksteps / 8));
        s = std::min(s, kMaxSplits);
        if ((int64_t)ksteps * (s - 1) <= (int64_t)40 * s) s = 1;
    } else if (split_k > 0) {
        s = split_k;
    } else if (nt < kCUs / 2) {
        // about one and a half blocks per CU; two for the smallest tiles; fewer for the 128-row
        // tiles of contraction-major operands, whose FP32 partial tiles are four times as large
        const int target = kTiles[t].bm * kTiles[t].bn <= 64 * 64 ? 512 : tn ? 160 : 384;
        s = std::max(1, (int)(target / nt));        // never more blocks than the target: the
                                                    // CUs that got one more would set the time
        s = std::min(s, std::max(1, ksteps / 8));  // at least eight stages per slice
        s = std::min(s, kMaxSplits);
    }
    s = std::max(1, std::min(s, ksteps));
    pl.splits = s;
    return pl;
}

// Upper bound of the workspace: one FP32 tile set per contraction slice.  (The MFMA kernel
// finishes its tiles itself only for an unsplit contraction, a row length that is a multiple
// of 16 and no FP32 / transposed output; otherwise it writes FP32 tiles and the finishing
// kernel takes over.)
static size_t plan_workspace(const Plan &pl, int64_t rows, int64_t cols) {
    if (!pl.mfma) return 0;
    return (size_t)pl.splits * (size_t)rows * (size_t)cols * sizeof(float);
}

}  // namespace mp8

extern "C" int mp8_gemm_num_tile_configs(void) { return mp8::kNumTiles; }

extern "C" int mp8_gemm_tile_config_name(int tile_config, char *buf, size_t buflen) {
    if (tile_config < 1 || tile_config > mp8::kNumTiles || !buf || buflen == 0) return -1;
    snprintf(buf, buflen, "%s", mp8::kTiles[tile_config - 1].name);
    return 0;
}

extern "C" int mp8_gemm_tile_config_lds_bytes(int tile_config, int epi) {
    if (tile_config < 1 || tile_config > mp8::kNumTiles || epi < 0 || epi > 2) return -1;
    hipFuncAttributes at;
    const mp8::TileConfig &tc = mp8::kTiles[tile_config - 1];
    const void *fn = tc.kernel[epi] ? (const void *)tc.kernel[epi] : (const void *)tc.kernel_tn[epi];
    if (fn == nullptr || hipFuncGetAttributes(&at, fn) != hipSuccess) return -1;
    return (int)at.sharedSizeBytes;
}

extern "C" size_t mp8_gemm_fp8_workspace_bytes_tuned(mp8_op op, int64_t M, int64_t N, int64_t K,
                                                     int tile_config, int split_k) {
    using namespace mp8;
    if (M <= 0 || N <= 0 || K <= 0 || (int)op < 0 || (int)op > 2) return 0;
    if (tile_config < 0 || tile_config > kNumTiles || split_k < 0) return 0;
    int64_t rows, cols, kc;
    op_dims(op, M, N, K, rows, cols, kc);
    // enough for every operand layout
    size_t need = 0;
    for (int layout : {0, 2, 3})
        need = std::max(need, plan_workspace(make_plan(rows, cols, kc, tile_config, split_k, layout), rows, cols));
    return need;
}

extern "C" mp8_status mp8_gemm_fp8_plan(mp8_op op, int64_t M, int64_t N, int64_t K, int flags,
                                        int tile_config, int split_k, int *tile_out,
                                        int *splits_out) {
    using namespace mp8;
    if (M <= 0 || N <= 0 || K <= 0 || (int)op < 0 || (int)op > 2) return MP8_ERR_INVALID_ARG;
    if (tile_config < 0 || tile_config > kNumTiles || split_k < 0) return MP8_ERR_INVALID_ARG;
    const bool atn = (flags & MP8_FLAG_A_CONTRACTION_MAJOR) != 0, btn = (flags & MP8_FLAG_B_CONTRACTION_MAJOR) != 0;
    if (atn && !btn) return MP8_ERR_UNSUPPORTED;
    int64_t rows, cols, kc;
    op_dims(op, M, N, K, rows, cols, kc);
    const Plan pl = make_plan(rows, cols, kc, tile_config, split_k, (atn ? 1 : 0) | (btn ? 2 : 0));
    if (tile_out) *tile_out = pl.mfma ? pl.tile + 1 : 0;
    if (splits_out) *splits_out = pl.splits;
    return MP8_OK;
}

extern "C" size_t mp8_gemm_fp8_workspace_bytes(mp8_op op, int64_t M, int64_t N, int64_t K) {
    return mp8_gemm_fp8_workspace_bytes_tuned(op, M, N, K, 0, 0);
}

namespace mp8 {

// Launch the MFMA kernel chosen by `pick` (indexed by EPI_*) for plan `pl`, and the finishing
// kernel when the epilogue cannot be fused.  `ga` carries the operands; its tiling, slicing and
// epilogue fields are filled in here.
static mp8_status launch_mfma(GemmArgs ga, const Epilogue &ep, const Plan &pl, int64_t kc,
                              void (*const pick[3])(const GemmArgs), void *workspace,
                              size_t workspace_bytes, hipStream_t s, const UpdateHook *upd = nullptr,
                              bool validate_only = false) {
    const int64_t rows = ep.rows, cols = ep.cols;
    const int acc_mode = ep.acc_mode;
    float *acc = ep.acc;
    uint8_t *out8 = ep.out8, *out8_t = ep.out8_t;
    // Fused epilogue or two passes?  (The master-weight update lives in the finishing pass.)
    const bool two_pass = pl.splits > 1 || (cols & 15) != 0 || acc_mode != 0 || out8_t != nullptr ||
                          upd != nullptr;
    float *partial = nullptr;
    Epilogue fin = ep;  // what the finishing kernel applies
    fin.want_codes = upd != nullptr;
    if (two_pass) {
        if (pl.splits == 1 && acc_mode == 1) {
            partial = acc;  // the tile goes straight into acc; the finishing kernel reads it there
            fin.acc = nullptr;
            fin.acc_mode = 0;
        } else {
            const size_t need = plan_workspace(pl, rows, cols);
            if (workspace == nullptr || workspace_bytes < need) return MP8_ERR_WORKSPACE;
            partial = (float *)workspace;
        }
    }
    const int64_t nblocks = (int64_t)pl.tiles_m * pl.tiles_n * pl.splits;
    if (nblocks > 0x7FFFFFFFLL) return MP8_ERR_UNSUPPORTED;
    if (validate_only) return MP8_OK;  // every check has passed; nothing is enqueued

    ga.rows = rows;
    ga.cols = cols;
    ga.ksteps = (int)(kc / BK);
    ga.splits = pl.splits;
    ga.tiles_m = pl.tiles_m;
    ga.tiles_n = pl.tiles_n;
    ga.div_tiles = make_fastdiv((uint32_t)(pl.tiles_m * pl.tiles_n));
    ga.div_band = make_fastdiv((uint32_t)(8 * pl.tiles_n));
    ga.div_tail = make_fastdiv((uint32_t)((pl.tiles_m & 7) ? (pl.tiles_m & 7) : 8));
    ga.div_tn = make_fastdiv((uint32_t)pl.tiles_n);
    ga.ks_per = ga.ksteps / pl.splits;
    ga.ks_extra = ga.ksteps % pl.splits;
    ga.partial = partial;
    ga.ep = ep;
    const int epi = two_pass ? EPI_PARTIAL
                             : (ep.sr || ep.sat || ep.stats != nullptr || out8 == nullptr) ? EPI_FULL
                                                                                            : EPI_RNE;
    const size_t dyn_lds = (size_t)kTiles[pl.tile].lds_per_stage * (size_t)ga.ksteps;
    hipLaunchKernelGGL(pick[epi], dim3((unsigned)nblocks), dim3(256), dyn_lds, s, ga);
    if (hipGetLastError() != hipSuccess) return MP8_ERR_HIP;
    if (two_pass) {
        const bool only_acc = fin.acc_mode == 0 && fin.out8 == nullptr && fin.out8_t == nullptr &&
                              fin.stats == nullptr && upd == nullptr;
        if (!only_acc) {
            const int64_t items = (cols & 3) == 0 ? rows * cols / 4 : rows * cols;
            int64_t blocks = std::min<int64_t>((items + 255) / 256, 256 * 16);
            const int states = upd ? upd->states : 0;
            hipLaunchKernelGGL(states == 2 ? splitk_finish_kernel<2>
                                           : states == 1 ? splitk_finish_kernel<1> : splitk_finish_kernel<0>,
                               dim3((unsigned)blocks), dim3(256), 0, s, (const float *)partial, pl.splits, fin,
                               upd ? *upd : UpdateHook{});
            if (hipGetLastError() != hipSuccess) return MP8_ERR_HIP;
        }
    }
    return MP8_OK;
}

}  // namespace mp8

namespace mp8 {

// mp8_gemm_fp8_tuned, optionally with the master-weight update applied to the rounded result
// (`upd`; only kernels with a finishing pass carry it: MP8_ERR_UNSUPPORTED otherwise).
static mp8_status gemm_impl(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                            const uint8_t *b, int64_t ldb, float alpha, float *acc, int acc_mode,
                            uint8_t *out8, uint8_t *out8_t, mp8_round round, int flags, uint64_t seed,
                            uint64_t offset, mp8_stats *stats, void *workspace, size_t workspace_bytes,
                            void *stream, int tile_config, int split_k, const UpdateHook *upd,
                            bool validate_only = false) {
    if ((int)op < 0 || (int)op > 2) return MP8_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0) return MP8_ERR_INVALID_ARG;
    if (round != MP8_RNE && round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (acc_mode < 0 || acc_mode > 2) return MP8_ERR_INVALID_ARG;
    if (tile_config < 0 || tile_config > kNumTiles || split_k < 0) return MP8_ERR_INVALID_ARG;
    int64_t rows, cols, kc;
    op_dims(op, M, N, K, rows, cols, kc);
    if (rows == 0 || cols == 0) return MP8_OK;
    if (acc_mode != 0 && acc == nullptr) return MP8_ERR_INVALID_ARG;
    if (kc > 0 && (!a || !b)) return MP8_ERR_INVALID_ARG;
    const bool atn = (flags & MP8_FLAG_A_CONTRACTION_MAJOR) != 0;
    const bool btn = (flags & MP8_FLAG_B_CONTRACTION_MAJOR) != 0;
    if (atn && !btn) return MP8_ERR_UNSUPPORTED;  // no kernel is built for this combination
    if (kc > 0 && (lda < (atn ? rows : kc) || ldb < (btn ? cols : kc))) return MP8_ERR_INVALID_ARG;
    if (rows > (INT64_MAX / 8) / cols) return MP8_ERR_UNSUPPORTED;
    if (((uintptr_t)acc | (uintptr_t)out8 | (uintptr_t)out8_t | (uintptr_t)workspace) & 15u)
        return MP8_ERR_ALIGNMENT;

    Epilogue ep{};
    ep.alpha = alpha;
    ep.acc = acc_mode ? acc : nullptr;
    ep.acc_mode = acc_mode;
    ep.out8 = out8;
    ep.out8_t = out8_t;
    ep.sr = round == MP8_SR;
    ep.sat = (flags & MP8_FLAG_SATURATE) ? 1 : 0;
    ep.seed = seed;
    ep.offset = offset;
    ep.stats = stats;
    ep.rows = rows;
    ep.cols = cols;
    hipStream_t s = (hipStream_t)stream;

    Plan pl = make_plan(rows, cols, kc, tile_config, split_k, (atn ? 1 : 0) | (btn ? 2 : 0));
    // the MFMA kernel wants 16-byte aligned rows and 32-bit offsets inside a 256-row tile
    const bool aligned = (((uintptr_t)a | (uintptr_t)b) & 15u) == 0 && (lda & 15) == 0 &&
                         (ldb & 15) == 0 && lda < (1 << 24) && ldb < (1 << 24);
    if (pl.mfma && !aligned) {
        if (tile_config > 0) return MP8_ERR_ALIGNMENT;
        pl.mfma = false;
        pl.splits = 1;
    }
    if (tile_config > 0 && !pl.mfma) return MP8_ERR_UNSUPPORTED;

    if (!pl.mfma || kc == 0) {
        if (upd != nullptr) return MP8_ERR_UNSUPPORTED;
        if (validate_only) return MP8_OK;
        int64_t blocks = std::min<int64_t>((rows * cols + 255) / 256, 1 << 20);
        hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a, lda, b,
                           ldb, kc, (atn ? 1 : 0) | (btn ? 2 : 0), ep);
        return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
    }

    GemmArgs ga{};
    ga.a = a;
    ga.b = b;
    ga.lda = lda;
    ga.ldb = ldb;
    const TileConfig &tc = kTiles[pl.tile];
    return launch_mfma(ga, ep, pl, kc, atn ? tc.kernel_tn : btn ? tc.kernel_bt : tc.kernel, workspace,
                       workspace_bytes, s, upd, validate_only);
}

// The checks of mp8_gemm_fp8 on these arguments without enqueuing anything: what a call made of
// several launches runs first, so that it is rejected as a whole or not at all.
static mp8_status gemm_validate(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                const uint8_t *b, int64_t ldb, float *acc, int acc_mode, uint8_t *out8,
                                uint8_t *out8_t, mp8_round round, int flags, void *workspace,
                                size_t workspace_bytes) {
    return gemm_impl(op, M, N, K, a, lda, b, ldb, 1.0f, acc, acc_mode, out8, out8_t, round, flags, 0, 0, nullptr,
                     workspace, workspace_bytes, nullptr, 0, 0, nullptr, true);
}

// Does the skip flag of a fused weight-gradient update live inside the statistics the same call
// accumulates into?  The finishing pass reads the flag when it starts and adds this gradient's
// Inf/NaN count when it ends, so such a flag would change under the pass that reads it; those
// calls run the weight gradient and the update as two launches instead, and the update then sees
// the final count.
static bool flag_inside_stats(const uint32_t *skip, const mp8_stats *stats) {
    if (skip == nullptr || stats == nullptr) return false;
    const uintptr_t f = (uintptr_t)skip, s0 = (uintptr_t)stats;
    return f + sizeof(uint32_t) > s0 && f < s0 + sizeof(mp8_stats);
}


// The master-weight update a finishing pass applies: plain SGD, or momentum SGD with L2
// regularisation when a velocity array is given (mp8_wgrad_adam_fp16_sr fills in ADAM's fields).
static UpdateHook make_update_hook(uint16_t *w16, uint8_t *w8_out, const uint32_t *skip, float lr,
                                   float inv_loss_scale, mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
                                   float *velocity = nullptr, float momentum = 0.0f, float weight_decay = 0.0f) {
    UpdateHook upd{};
    upd.w16 = w16;
    upd.w8_out = w8_out;
    upd.skip = skip;
    upd.neg_lr = -lr;
    upd.inv_scale = inv_loss_scale;
    upd.sr = w_round == MP8_SR;
    upd.seed = w_seed;
    upd.offset = w_offset;
    upd.states = velocity != nullptr ? 1 : 0;
    upd.state0 = velocity;
    upd.mu = momentum;
    upd.wd = weight_decay;
    return upd;
}

// Where the 8-bit weight gradient goes when the update is cheaper as a launch of its own: a
// weight-gradient GEMM that runs unsplit rounds in its own epilogue, and forcing a finishing pass
// on it just to carry the update would write and re-read the whole FP32 result (measured: 1024 x
// 4096 from 16384 tokens 91 against 77 us).  Then the codes go to g8_out, or to the workspace if
// the caller keeps no gradient, and the stand-alone update kernel follows.  Null: use the
// finishing pass.
static uint8_t *codes_for_separate_update(int64_t M, int64_t N, int64_t K, int flags, uint8_t *g8_out,
                                          void *workspace, size_t workspace_bytes) {
    const bool atn = (flags & MP8_FLAG_A_CONTRACTION_MAJOR) != 0, btn = (flags & MP8_FLAG_B_CONTRACTION_MAJOR) != 0;
    if ((atn && !btn) || (N & 15) != 0 || K > (INT64_MAX / 8) / std::max<int64_t>(N, 1)) return nullptr;
    const Plan pl = make_plan(K, N, M, 0, 0, (atn ? 1 : 0) | (btn ? 2 : 0));
    if (!pl.mfma || pl.splits != 1) return nullptr;
    if (g8_out != nullptr) return g8_out;
    return workspace != nullptr && workspace_bytes >= (size_t)(K * N) ? (uint8_t *)workspace : nullptr;
}
}  // namespace mp8

extern "C" mp8_status mp8_gemm_fp8_tuned(mp8_op op, int64_t M, int64_t N, int64_t K,
                                         const uint8_t *a, int64_t lda, const uint8_t *b,
                                         int64_t ldb, float alpha, float *acc, int acc_mode,
                                         uint8_t *out8, uint8_t *out8_t, mp8_round round,
                                         int flags, uint64_t seed, uint64_t offset,
                                         mp8_stats *stats, void *workspace,
                                         size_t workspace_bytes, void *stream, int tile_config,
                                         int split_k) {
    return mp8::gemm_impl(op, M, N, K, a, lda, b, ldb, alpha, acc, acc_mode, out8, out8_t, round, flags,
                          seed, offset, stats, workspace, workspace_bytes, stream, tile_config, split_k,
                          nullptr);
}

namespace mp8 {

// Weight gradient, its rounding, and a master-weight update of the rounded codes (Figure 1b): the
// body the three optimizer variants share.  `hook` is the rule as the finishing pass applies it,
// `update_from(codes)` launches the same rule's stand-alone kernel on codes in memory.  Three ways,
// all with the same results: the GEMM with its own epilogue followed by the update kernel (unsplit
// contractions, any-shape kernel, and a skip flag that lives inside `stats` -- see
// flag_inside_stats), or the update inside the finishing pass of a split contraction.  Whatever
// can be checked is checked before the first launch.
template <class UpdateFrom>
static mp8_status wgrad_with_update(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                    const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                    mp8_round g_round, int flags, uint64_t g_seed, uint64_t g_offset,
                                    mp8_stats *stats, const UpdateHook &hook, void *workspace,
                                    size_t workspace_bytes, void *stream, UpdateFrom update_from) {
    auto two_launches = [&](uint8_t *codes, void *ws, size_t ws_bytes) -> mp8_status {
        const mp8_status sv = gemm_validate(MP8_WGRAD, M, N, K, a, lda, b, ldb, nullptr, 0, codes, nullptr,
                                            g_round, flags, ws, ws_bytes);
        if (sv != MP8_OK) return sv;
        const mp8_status sg = mp8_gemm_fp8(MP8_WGRAD, M, N, K, a, lda, b, ldb, alpha, nullptr, 0, codes, nullptr,
                                           g_round, flags, g_seed, g_offset, stats, ws, ws_bytes, stream);
        if (sg != MP8_OK) return sg;
        return update_from(codes);
    };
    if (uint8_t *codes = codes_for_separate_update(M, N, K, flags, g8_out, workspace, workspace_bytes))
        return two_launches(codes, nullptr, 0);
    if (flag_inside_stats(hook.skip, stats))
        return g8_out != nullptr ? two_launches(g8_out, workspace, workspace_bytes) : MP8_ERR_INVALID_ARG;
    const mp8_status st = gemm_impl(MP8_WGRAD, M, N, K, a, lda, b, ldb, alpha, nullptr, 0, g8_out, nullptr,
                                    g_round, flags, g_seed, g_offset, stats, workspace, workspace_bytes,
                                    stream, 0, 0, &hook);
    if (st != MP8_ERR_UNSUPPORTED || g8_out == nullptr) return st;
    // shapes that only the any-shape kernel takes: two launches through the 8-bit gradient
    return two_launches(g8_out, workspace, workspace_bytes);
}

}  // namespace mp8

extern "C" mp8_status mp8_wgrad_update_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a,
                                               int64_t lda, const uint8_t *b, int64_t ldb, float alpha,
                                               uint8_t *g8_out, mp8_round g_round, int flags,
                                               uint64_t g_seed, uint64_t g_offset, mp8_stats *stats,
                                               uint16_t *w16, float lr, float inv_loss_scale,
                                               mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
                                               const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                               void *workspace, size_t workspace_bytes, void *stream) {
    using namespace mp8;
    if (M < 0 || N < 0 || K < 0) return MP8_ERR_INVALID_ARG;
    if (w_round != MP8_RNE && w_round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (K == 0 || N == 0) return MP8_OK;
    if (!w16) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)w8_out) & 15u) return MP8_ERR_ALIGNMENT;
    const UpdateHook upd = make_update_hook(w16, w8_out, skip_if_nonzero, lr, inv_loss_scale, w_round, w_seed, w_offset);
    return wgrad_with_update(M, N, K, a, lda, b, ldb, alpha, g8_out, g_round, flags, g_seed, g_offset, stats, upd,
                             workspace, workspace_bytes, stream, [&](const uint8_t *codes) {
        return mp8_sgd_update_fp16_sr(w16, codes, K * N, lr, inv_loss_scale, w_round, w_seed, w_offset,
                                      skip_if_nonzero, w8_out, nullptr, stream);
    });
}

extern "C" mp8_status mp8_wgrad_momentum_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                                 const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                                 mp8_round g_round, int flags, uint64_t g_seed,
                                                 uint64_t g_offset, mp8_stats *stats, uint16_t *w16,
                                                 float *velocity, float lr, float inv_loss_scale,
                                                 float momentum, float weight_decay, mp8_round w_round,
                                                 uint64_t w_seed, uint64_t w_offset,
                                                 const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                                 void *workspace, size_t workspace_bytes, void *stream) {
    using namespace mp8;
    if (M < 0 || N < 0 || K < 0) return MP8_ERR_INVALID_ARG;
    if (w_round != MP8_RNE && w_round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (K == 0 || N == 0) return MP8_OK;
    if (!w16 || !velocity) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)w8_out | (uintptr_t)velocity) & 15u) return MP8_ERR_ALIGNMENT;
    const UpdateHook upd = make_update_hook(w16, w8_out, skip_if_nonzero, lr, inv_loss_scale, w_round, w_seed, w_offset,
                                            velocity, momentum, weight_decay);
    return wgrad_with_update(M, N, K, a, lda, b, ldb, alpha, g8_out, g_round, flags, g_seed, g_offset, stats, upd,
                             workspace, workspace_bytes, stream, [&](const uint8_t *codes) {
        return mp8_sgd_momentum_fp16_sr(w16, velocity, codes, K * N, lr, inv_loss_scale, momentum, weight_decay,
                                        w_round, w_seed, w_offset, skip_if_nonzero, w8_out, nullptr, stream);
    });
}

extern "C" mp8_status mp8_wgrad_adam_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                             const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                             mp8_round g_round, int flags, uint64_t g_seed, uint64_t g_offset,
                                             mp8_stats *stats, uint16_t *w16, float *m, float *v, float lr,
                                             float inv_loss_scale, float beta1, float beta2, float eps,
                                             float weight_decay, int64_t step, mp8_round w_round,
                                             uint64_t w_seed, uint64_t w_offset,
                                             const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                             void *workspace, size_t workspace_bytes, void *stream) {
    using namespace mp8;
    if (M < 0 || N < 0 || K < 0 || step < 1) return MP8_ERR_INVALID_ARG;
    if (w_round != MP8_RNE && w_round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (K == 0 || N == 0) return MP8_OK;
    if (!w16 || !m || !v) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)w8_out | (uintptr_t)m | (uintptr_t)v) & 15u) return MP8_ERR_ALIGNMENT;
    UpdateHook upd = make_update_hook(w16, w8_out, skip_if_nonzero, lr, inv_loss_scale, w_round, w_seed, w_offset);
    upd.states = 2;
    upd.state0 = m;
    upd.state1 = v;
    upd.wd = weight_decay;
    upd.b1 = beta1;
    upd.b2 = beta2;
    upd.omb1 = 1.0f - beta1;
    upd.omb2 = 1.0f - beta2;
    // bias corrections as in mp8_adam_fp16_sr: the powers in double, the result as FP32
    upd.c1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    upd.c2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    upd.eps = eps;
    return wgrad_with_update(M, N, K, a, lda, b, ldb, alpha, g8_out, g_round, flags, g_seed, g_offset, stats, upd,
                             workspace, workspace_bytes, stream, [&](const uint8_t *codes) {
        return mp8_adam_fp16_sr(w16, m, v, codes, K * N, lr, inv_loss_scale, beta1, beta2, eps, weight_decay, step,
                                w_round, w_seed, w_offset, skip_if_nonzero, w8_out, nullptr, stream);
    });
}

extern "C" mp8_status mp8_gemm_fp8(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a,
                                   int64_t lda, const uint8_t *b, int64_t ldb, float alpha,
                                   float *acc, int acc_mode, uint8_t *out8, uint8_t *out8_t,
                                   mp8_round round, int flags, uint64_t seed, uint64_t offset,
                                   mp8_stats *stats, void *workspace, size_t workspace_bytes,
                                   void *stream) {
    return mp8_gemm_fp8_tuned(op, M, N, K, a, lda, b, ldb, alpha, acc, acc_mode, out8, out8_t,
                              round, flags, seed, offset, stats, workspace, workspace_bytes,
                              stream, 0, 0);
}

// ---------------------------------------------------------------------------------------
// mp8_gemm_fp8 for callers that cannot allocate: the scratch of the two-pass paths (FP32 tiles of
// the contraction slices, unfused epilogues) lives in a static device array of this library.
namespace mp8 {

constexpr size_t kStaticScratchBytes = (size_t)MP8_STATIC_SCRATCH_BYTES;
// Every GPU the library runs on holds its own copy of this array, at an address of its own, until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels get
// the device address looked up below, never the name.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, once looked up
static std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device).
static mp8_status static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MP8_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return MP8_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MP8_OK;
}

}  // namespace mp8

extern "C" size_t mp8_static_scratch_bytes(void) { return mp8::kStaticScratchBytes; }

extern "C" mp8_status mp8_gemm_fp8_static(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a,
                                          int64_t lda, const uint8_t *b, int64_t ldb, float alpha,
                                          float *acc, int acc_mode, uint8_t *out8, uint8_t *out8_t,
                                          mp8_round round, int flags, uint64_t seed, uint64_t offset,
                                          mp8_stats *stats, void *stream) {
    using namespace mp8;
    // the same bound the workspace query gives the callers of mp8_gemm_fp8
    if (M > 0 && N > 0 && K > 0 && (int)op >= 0 && (int)op <= 2 &&
        mp8_gemm_fp8_workspace_bytes(op, M, N, K) > kStaticScratchBytes)
        return MP8_ERR_WORKSPACE;
    void *ws = nullptr;
    const mp8_status ss = static_scratch(&ws);
    if (ss != MP8_OK) return ss;
    // Nothing in the scratch has to start at zero: every FP32 tile element the finishing pass
    // reads has been written by this call's first kernel.
    return gemm_impl(op, M, N, K, a, lda, b, ldb, alpha, acc, acc_mode, out8, out8_t, round, flags, seed,
                     offset, stats, ws, kStaticScratchBytes, stream, 0, 0, nullptr);
}

// ---------------------------------------------------------------------------------------
// GEMMs that quantise their own FP32 operand

extern "C" mp8_status mp8_quantize_gemm_fwd_fp8(int64_t M, int64_t N, int64_t K, const float *x,
                                                float x_scale, mp8_round x_round, int x_flags,
                                                uint64_t x_seed, uint64_t x_offset, mp8_stats *x_stats,
                                                uint8_t *x8_out, const uint8_t *w8, int64_t ldw,
                                                float alpha, float *acc, int acc_mode, uint8_t *out8,
                                                uint8_t *out8_t, mp8_round round, int flags,
                                                uint64_t seed, uint64_t offset, mp8_stats *stats,
                                                void *workspace, size_t workspace_bytes, void *stream) {
    using namespace mp8;
    if (M < 0 || N < 0 || K < 0) return MP8_ERR_INVALID_ARG;
    if ((x_round != MP8_RNE && x_round != MP8_SR) || (round != MP8_RNE && round != MP8_SR))
        return MP8_ERR_INVALID_ARG;
    if (acc_mode < 0 || acc_mode > 2) return MP8_ERR_INVALID_ARG;
    if (M == 0) return MP8_OK;  // nothing to round, nothing to multiply
    if (acc_mode != 0 && acc == nullptr && N > 0) return MP8_ERR_INVALID_ARG;
    if (K > 0 && (!x || !x8_out)) return MP8_ERR_INVALID_ARG;
    if (N > 0 && K > 0 && (!w8 || ldw < N)) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)x | (uintptr_t)x8_out | (uintptr_t)acc | (uintptr_t)out8 | (uintptr_t)out8_t) & 15u)
        return MP8_ERR_ALIGNMENT;
    const bool fused = N >= 16 && N <= 128 && (N & 15) == 0 && K > 0 && (K & (BK - 1)) == 0 &&
                       ((uintptr_t)w8 & 15u) == 0 && (ldw & 15) == 0 && ldw < (1 << 24) &&
                       M <= (INT64_MAX / 8) / K && (M + 63) / 64 <= 0x7FFFFFFFLL;
    if (!fused) {
        // any other shape: the two calls this one stands for (the second one's checks first, so
        // that a rejected call has enqueued nothing)
        const int gflags = (flags & MP8_FLAG_SATURATE) | MP8_FLAG_B_CONTRACTION_MAJOR;
        if (N > 0 && K > 0) {
            const mp8_status sv = gemm_validate(MP8_FWD, M, N, K, x8_out, K, w8, ldw, acc, acc_mode, out8, out8_t,
                                                round, gflags, workspace, workspace_bytes);
            if (sv != MP8_OK) return sv;
        }
        const mp8_status sq = mp8_quantize_e5m2(x, 0, x8_out, nullptr, M, K, x_scale, x_round, x_flags,
                                                x_seed, x_offset, x_stats, stream);
        if (sq != MP8_OK) return sq;
        return mp8_gemm_fp8(MP8_FWD, M, N, K, x8_out, K, w8, ldw, alpha, acc, acc_mode, out8, out8_t,
                            round, gflags, seed, offset, stats, workspace, workspace_bytes, stream);
    }
    GemmArgs ga{};
    ga.b = w8;
    ga.ldb = ldw;
    ga.rows = M;
    ga.cols = N;
    ga.ksteps = (int)(K / BK);
    ga.splits = 1;
    Epilogue &ep = ga.ep;
    ep.alpha = alpha;
    ep.acc = acc_mode ? acc : nullptr;
    ep.acc_mode = acc_mode;
    ep.out8 = out8;
    ep.out8_t = out8_t;
    ep.sr = round == MP8_SR;
    ep.sat = (flags & MP8_FLAG_SATURATE) ? 1 : 0;
    ep.seed = seed;
    ep.offset = offset;
    ep.stats = stats;
    ep.rows = M;
    ep.cols = N;
    QuantArgs qa{};
    qa.x = x;
    qa.x8 = x8_out;
    qa.scale = x_scale;
    qa.sr = x_round == MP8_SR;
    qa.sat = (x_flags & MP8_FLAG_SATURATE) ? 1 : 0;
    qa.seed = x_seed;
    qa.offset = x_offset;
    qa.stats = x_stats;
    const bool plain = acc_mode == 0 && out8_t == nullptr && !ep.sr && !ep.sat && stats == nullptr &&
                       out8 != nullptr;
    const bool qplain = !qa.sr && !qa.sat && x_stats == nullptr;
    // 128 rows per workgroup once that still gives every other CU a workgroup
    const bool tall = (M + 127) / 128 >= 128;
    void (*kernel)(const GemmArgs, const QuantArgs);
    if (tall)
        kernel = plain ? (qplain ? gemm_qfwd_kernel<EPI_RNE, true, 128> : gemm_qfwd_kernel<EPI_RNE, false, 128>)
                       : (qplain ? gemm_qfwd_kernel<EPI_FULL, true, 128> : gemm_qfwd_kernel<EPI_FULL, false, 128>);
    else
        kernel = plain ? (qplain ? gemm_qfwd_kernel<EPI_RNE, true, 64> : gemm_qfwd_kernel<EPI_RNE, false, 64>)
                       : (qplain ? gemm_qfwd_kernel<EPI_FULL, true, 64> : gemm_qfwd_kernel<EPI_FULL, false, 64>);
    const int bm = tall ? 128 : 64;
    hipLaunchKernelGGL(kernel, dim3((unsigned)((M + bm - 1) / bm)), dim3(4 * bm + 256), 0,
                       (hipStream_t)stream, ga, qa);
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}

// ---------------------------------------------------------------------------------------
// 3x3 convolution as an implicit GEMM on zero-padded channels-last tensors
// ---------------------------------------------------------------------------------------
namespace mp8 {

struct ConvDims {
    int64_t rows, cols, kc;  // of the implicit GEMM
    int64_t lda, ldb;
};

static bool conv_dims(mp8_op op, int64_t prows, int64_t Ci, int64_t Co, ConvDims &d) {
    switch (op) {
        case MP8_FWD: d = {prows, Co, 9 * Ci, Ci, Co}; return true;
        case MP8_BWD_DATA: d = {prows, Ci, 9 * Co, Co, Co}; return true;
        case MP8_WGRAD: d = {9 * Ci, Co, prows, Ci, Co}; return true;
    }
    return false;
}

// Stages of the implicit GEMM's contraction: whole stages of 128, the last one starting 64 early
// when forward / backward data contract over an odd number of 64-channel units.
static int64_t conv_kc_stages(const ConvDims &d) { return (d.kc + BK - 1) / BK * BK; }

static Plan conv_plan(mp8_op op, const ConvDims &d, int64_t Ci) {
    // the tile shapes built for contraction-major operands are the ones built for convolutions
    const int64_t kc = conv_kc_stages(d);
    Plan pl = make_plan(d.rows, d.cols, kc, 0, 0, 3, true);
    // a tile row of the weight gradient must not straddle two taps
    if (pl.mfma && op == MP8_WGRAD && (Ci % kTiles[pl.tile].bm) != 0)
        pl = make_plan(d.rows, d.cols, kc, ((Ci & 127) == 0 ? T128x128s2 : T64x64s2) + 1, 0, 3, true);
    // forward and backward data have one tile row per 128 pixels and few tile columns: the
    // 128-row tile keeps the re-reads of the weights low; it is also the tile whose kernels are
    // built for stages that span two taps (contracted channels an odd multiple of 64)
    if (pl.mfma && op != MP8_WGRAD && (kTiles[pl.tile].bm < 128 || (d.kc / 9 / 64) % 2 != 0))
        pl = make_plan(d.rows, d.cols, kc, T128x128s2 + 1, 0, 3, true);
    // ... and for 64 output columns a 128x64 tile of the same kind (tile geometry and slices as
    // for the row-major kernel of that shape)
    if (pl.mfma && op != MP8_WGRAD && (d.kc / 9 / 64) % 2 != 0 && d.cols == 64)
        pl = make_plan(d.rows, d.cols, kc, T128x64s2 + 1, 0, 0, true);
    return pl;
}

// Forward / backward data with the contracted channel count an odd multiple of 64: [op][EPI_*]
static void (*const kConvHalves[2][3])(const GemmArgs) = {
    {gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_PARTIAL, false, true, 4>,
     gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_RNE, false, true, 4>,
     gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_FULL, false, true, 4>},
    {gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_PARTIAL, false, false, 5>,
     gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_RNE, false, false, 5>,
     gemm_mfma_kernel<128, 128, 2, 2, 2, 2, EPI_FULL, false, false, 5>}};
// the same for 64 output columns
static void (*const kConvHalves64[2][3])(const GemmArgs) = {
    {gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_PARTIAL, false, true, 4>,
     gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_RNE, false, true, 4>,
     gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_FULL, false, true, 4>},
    {gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_PARTIAL, false, false, 5>,
     gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_RNE, false, false, 5>,
     gemm_mfma_kernel<128, 64, 4, 1, 2, 3, EPI_FULL, false, false, 5>}};

}  // namespace mp8

extern "C" size_t mp8_conv3x3_fp8_workspace_bytes(mp8_op op, int64_t B, int64_t H, int64_t W,
                                                  int64_t Ci, int64_t Co, int64_t prows) {
    using namespace mp8;
    ConvDims d;
    if (B <= 0 || H <= 0 || W <= 0 || Ci <= 0 || Co <= 0 || prows <= 0) return 0;
    if (!conv_dims(op, prows, Ci, Co, d)) return 0;
    return plan_workspace(conv_plan(op, d, Ci), d.rows, d.cols);
}

namespace mp8 {

// mp8_conv3x3_fp8, optionally (weight gradient only) with the master-weight update applied to
// the rounded result by the finishing pass.
static mp8_status conv_impl(mp8_op op, int64_t B, int64_t H, int64_t W, int64_t Ci, int64_t Co,
                            int64_t prows, const uint8_t *a, const uint8_t *b, float alpha, float *acc,
                            int acc_mode, uint8_t *out8, mp8_round round, int flags, uint64_t seed,
                            uint64_t offset, mp8_stats *stats, void *workspace, size_t workspace_bytes,
                            void *stream, const UpdateHook *upd) {
    ConvDims d;
    if (B < 0 || H < 0 || W < 0 || Ci < 0 || Co < 0 || prows < 0) return MP8_ERR_INVALID_ARG;
    if (!conv_dims(op, prows, Ci, Co, d)) return MP8_ERR_INVALID_ARG;
    if (round != MP8_RNE && round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (acc_mode < 0 || acc_mode > 2) return MP8_ERR_INVALID_ARG;
    if (flags & ~MP8_FLAG_SATURATE) return MP8_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || W == 0 || Ci == 0 || Co == 0) return MP8_OK;
    const int64_t img = (H + 2) * (W + 2);
    if (B > (int64_t)0x7FFFFFFF / img || prows < B * img || prows > 0x7FFFFFFF) return MP8_ERR_INVALID_ARG;
    if (!a || !b || (acc_mode != 0 && !acc)) return MP8_ERR_INVALID_ARG;
    // whole 64-byte halves of a stage per tap, whole tiles per tap of the weight gradient; lane
    // offsets (a tile's rows, a filter row's shift, a tap's weight slab) stay within 32 bits
    if ((Ci & 63) != 0 || (Co & 63) != 0 || Ci >= (1 << 15) || Co >= (1 << 15) || W >= (1 << 15))
        return MP8_ERR_UNSUPPORTED;
    if (op == MP8_WGRAD && (prows & 127) != 0) return MP8_ERR_UNSUPPORTED;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)acc | (uintptr_t)out8 | (uintptr_t)workspace) & 15u)
        return MP8_ERR_ALIGNMENT;
    const Plan pl = conv_plan(op, d, Ci);
    if (!pl.mfma) return MP8_ERR_UNSUPPORTED;

    Epilogue ep{};
    ep.alpha = alpha;
    ep.acc = acc_mode ? acc : nullptr;
    ep.acc_mode = acc_mode;
    ep.out8 = out8;
    ep.sr = round == MP8_SR;
    ep.sat = (flags & MP8_FLAG_SATURATE) ? 1 : 0;
    ep.seed = seed;
    ep.offset = offset;
    ep.stats = stats;
    ep.rows = d.rows;
    ep.cols = d.cols;
    if (op != MP8_WGRAD) {
        ep.mask = 1;
        ep.hh = (int)(H + 2);
        ep.valid_rows = B * img;
        ep.div_img = make_fastdiv((uint32_t)img);
        ep.div_w2 = make_fastdiv((uint32_t)(W + 2));
    }
    GemmArgs ga{};
    ga.a = a;
    ga.b = b;
    ga.lda = d.lda;
    ga.ldb = d.ldb;
    ga.cv.w2 = (int)(W + 2);
    ga.cv.units_per_tap = (int)((op == MP8_BWD_DATA ? Co : Ci) / 64);
    ga.cv.div_cpb = make_fastdiv((uint32_t)ga.cv.units_per_tap);
    ga.cv.odd_units = op != MP8_WGRAD && (d.kc % BK) != 0;
    ga.cv.b_tap_stride = Ci * Co;
    ga.cv.div_ci = make_fastdiv((uint32_t)Ci);
    const bool halves = op != MP8_WGRAD && (ga.cv.units_per_tap & 1) != 0;
    if (halves && pl.tile != T128x128s2 && pl.tile != T128x64s2) return MP8_ERR_UNSUPPORTED;
    return launch_mfma(ga, ep, pl, conv_kc_stages(d),
                       !halves ? kTiles[pl.tile].kernel_conv[(int)op]
                               : pl.tile == T128x64s2 ? kConvHalves64[(int)op] : kConvHalves[(int)op],
                       workspace, workspace_bytes,
                       (hipStream_t)stream, upd);
}

}  // namespace mp8

extern "C" mp8_status mp8_conv3x3_fp8(mp8_op op, int64_t B, int64_t H, int64_t W, int64_t Ci,
                                      int64_t Co, int64_t prows, const uint8_t *a,
                                      const uint8_t *b, float alpha, float *acc, int acc_mode,
                                      uint8_t *out8, mp8_round round, int flags, uint64_t seed,
                                      uint64_t offset, mp8_stats *stats, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    return mp8::conv_impl(op, B, H, W, Ci, Co, prows, a, b, alpha, acc, acc_mode, out8, round, flags, seed,
                          offset, stats, workspace, workspace_bytes, stream, nullptr);
}

extern "C" mp8_status mp8_conv3x3_wgrad_update_fp16_sr(
    int64_t B, int64_t H, int64_t W, int64_t Ci, int64_t Co, int64_t prows, const uint8_t *x8,
    const uint8_t *e8, float alpha, uint8_t *g8_out, mp8_round g_round, int flags, uint64_t g_seed,
    uint64_t g_offset, mp8_stats *stats, uint16_t *w16, float lr, float inv_loss_scale,
    mp8_round w_round, uint64_t w_seed, uint64_t w_offset, const uint32_t *skip_if_nonzero,
    uint8_t *w8_out, void *workspace, size_t workspace_bytes, void *stream) {
    using namespace mp8;
    if (w_round != MP8_RNE && w_round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || W == 0 || Ci == 0 || Co == 0) return MP8_OK;
    if (!w16) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)w8_out) & 15u) return MP8_ERR_ALIGNMENT;
    if (flag_inside_stats(skip_if_nonzero, stats)) {
        // the flag is still being counted while the finishing pass would read it: two launches
        if (g8_out == nullptr) return MP8_ERR_INVALID_ARG;
        const mp8_status sg = conv_impl(MP8_WGRAD, B, H, W, Ci, Co, prows, x8, e8, alpha, nullptr, 0, g8_out, g_round,
                                        flags, g_seed, g_offset, stats, workspace, workspace_bytes, stream, nullptr);
        if (sg != MP8_OK) return sg;
        return mp8_sgd_update_fp16_sr(w16, g8_out, 9 * Ci * Co, lr, inv_loss_scale, w_round, w_seed, w_offset,
                                      skip_if_nonzero, w8_out, nullptr, stream);
    }
    UpdateHook upd = make_update_hook(w16, w8_out, skip_if_nonzero, lr, inv_loss_scale, w_round, w_seed, w_offset);
    return conv_impl(MP8_WGRAD, B, H, W, Ci, Co, prows, x8, e8, alpha, nullptr, 0, g8_out, g_round, flags,
                     g_seed, g_offset, stats, workspace, workspace_bytes, stream, &upd);
}

extern "C" mp8_status mp8_conv3x3_wgrad_momentum_fp16_sr(
    int64_t B, int64_t H, int64_t W, int64_t Ci, int64_t Co, int64_t prows, const uint8_t *x8,
    const uint8_t *e8, float alpha, uint8_t *g8_out, mp8_round g_round, int flags, uint64_t g_seed,
    uint64_t g_offset, mp8_stats *stats, uint16_t *w16, float *velocity, float lr, float inv_loss_scale,
    float momentum, float weight_decay, mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
    const uint32_t *skip_if_nonzero, uint8_t *w8_out, void *workspace, size_t workspace_bytes,
    void *stream) {
    using namespace mp8;
    if (w_round != MP8_RNE && w_round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || W == 0 || Ci == 0 || Co == 0) return MP8_OK;
    if (!w16 || !velocity) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)w8_out | (uintptr_t)velocity) & 15u) return MP8_ERR_ALIGNMENT;
    if (flag_inside_stats(skip_if_nonzero, stats)) {
        if (g8_out == nullptr) return MP8_ERR_INVALID_ARG;
        const mp8_status sg = conv_impl(MP8_WGRAD, B, H, W, Ci, Co, prows, x8, e8, alpha, nullptr, 0, g8_out, g_round,
                                        flags, g_seed, g_offset, stats, workspace, workspace_bytes, stream, nullptr);
        if (sg != MP8_OK) return sg;
        return mp8_sgd_momentum_fp16_sr(w16, velocity, g8_out, 9 * Ci * Co, lr, inv_loss_scale, momentum,
                                        weight_decay, w_round, w_seed, w_offset, skip_if_nonzero, w8_out, nullptr,
                                        stream);
    }
    UpdateHook upd = make_update_hook(w16, w8_out, skip_if_nonzero, lr, inv_loss_scale, w_round, w_seed, w_offset,
                                      velocity, momentum, weight_decay);
    return conv_impl(MP8_WGRAD, B, H, W, Ci, Co, prows, x8, e8, alpha, nullptr, 0, g8_out, g_round, flags,
                     g_seed, g_offset, stats, workspace, workspace_bytes, stream, &upd);
}
