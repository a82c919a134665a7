// GEMM kernel for small outputs with long contractions: the contraction is divided among the
// waves of a workgroup.
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

// Small output, long contraction (weight gradients, skinny layers): the contraction is divided
// among the four WAVES of a workgroup as well.  In the general kernel a 64x64 tile gives each
// wave one 32x32 MFMA per half stage behind a workgroup barrier, and every stage costs a chain
// of latencies (load, barrier, LDS read, MFMA) with nothing to overlap them.  Here every wave
// computes the whole 64x64 tile (four MFMAs per half stage, each fragment used twice) for every
// fourth stage of the workgroup's slice, from a two-stage ring of its own (2 x 16 KB) that it
// fills with its own direct loads and waits for with its own counter: no barrier inside the
// loop, and eight stage loads in flight per CU.  At the end the four FP32 tiles meet in LDS and
// are added in wave order; each thread then owns sixteen consecutive columns of one row for
// the epilogue.  Operand layouts and slab images as in the general kernel (ATN / BTN:
// contraction-major).  CONV = 3: the weight gradient of the 3x3 convolution (tap shift per tile
// row), else 0.  BM = 32 / BN = 32 (row-major operand only): half the tile rows / columns, for
// outputs with so few 64x64 tiles that most CUs would idle while the busy ones wait for their
// own loads (a CU takes 64 bytes per clock however few of them work).
template <int EPI, bool ATN, bool BTN, int CONV, int BM = 64, int BN = 64>
__global__ __launch_bounds__(256, 1) void gemm_wavek_kernel(const GemmArgs p) {
    static_assert(CONV == 0 || (CONV == 3 && ATN && BTN), "plain or convolution weight gradient");
    static_assert(BTN || !ATN, "a alone contraction-major is not built");
    static_assert(BM == 64 || (BM == 32 && !ATN), "the 32-row tile takes a row-major a");
    static_assert(BN == 64 || (BN == 32 && !BTN), "the 32-column tile takes a row-major b");
    constexpr int MI = BM / 32, NJ = BN / 32;  // 32x32 accumulator tiles along rows and columns
    constexpr int QA = BM / 8, QB = BN / 8;    // direct loads per stage and operand (eight rows each)
    constexpr int SLAB_A = BM * BK;         // BM rows of 128 bytes, or 128 contraction rows of 64
    constexpr int SLAB = BN * BK;           // b
    constexpr int STAGE = SLAB_A + SLAB;    // a, then b
    constexpr int WAVE_LDS = 2 * STAGE;     // ring of two stages per wave
    constexpr int RED_LD = BN + 4;          // floats per row of a tile parked for the reduction
    static_assert(4 * BM * RED_LD * 4 <= 4 * WAVE_LDS, "reduction buffers fit in the rings");
    __shared__ __attribute__((aligned(1024))) uint8_t lds[4 * WAVE_LDS];

    int split, tm, tn;
    map_block(p, split, tm, tn);
    split = __builtin_amdgcn_readfirstlane(split);
    tm = __builtin_amdgcn_readfirstlane(tm);
    tn = __builtin_amdgcn_readfirstlane(tn);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int per = p.ks_per, extra = p.ks_extra;
    const int ks_begin = split * per + (split < extra ? split : extra);
    const int ks_count = per + (split < extra ? 1 : 0);
    // this wave's stages: ks_begin + wave, + 4, + 8, ...
    const int mine = __builtin_amdgcn_readfirstlane(ks_count > wave ? (ks_count - wave + 3) >> 2 : 0);

    const int64_t a_kstep = ATN ? (int64_t)BK * p.lda : BK, b_kstep = BTN ? (int64_t)BK * p.ldb : BK;
    const uint8_t *a_origin;
    if constexpr (CONV == 3) {
        uint32_t ci0;
        const uint32_t tap = fastdiv((uint32_t)row0, p.cv.div_ci, ci0);
        const int r = (int)((tap * 11u) >> 5);
        const int shift = (r - 1) * p.cv.w2 + ((int)tap - 3 * r - 1);
        a_origin = p.a + (int64_t)shift * p.lda + ci0;
    } else {
        a_origin = ATN ? p.a + row0 : p.a + row0 * p.lda;
    }
    const uint8_t *b_origin = BTN ? p.b + col0 : p.b + col0 * p.ldb;
    const uint8_t *a_tile = uniform_ptr(a_origin + (int64_t)(ks_begin + wave) * a_kstep);
    const uint8_t *b_tile = uniform_ptr(b_origin + (int64_t)(ks_begin + wave) * b_kstep);
    // Direct loads, eight per operand and stage.  Row-major operand: load q brings tile rows
    // 8q .. 8q+7, lane i lands at (row i/8, slot i%8) and fetches chunk (i%8) ^ ((row >> 1) & 7);
    // rows beyond the matrix are clamped to its last row.  Contraction-major operand: load q
    // brings contraction rows 16q .. 16q+15 of 64 bytes, lane i lands at (row i/4, slot i%4) and
    // fetches the chunk that belongs there under the swizzle of the narrow slabs; chunks that
    // would start beyond the matrix are clamped to its last 16 rows.  (Clamped data is never
    // stored.)
    auto lane_offsets = [&](bool km, int64_t first, int64_t limit, int64_t ld, uint32_t off[8]) {
        if (km) {
            const int chunk = (lane & 3) ^ (((lane >> 4) & 1) << 1);
            int64_t m = 16 * chunk;
            m = first + m + 16 <= limit ? m : limit - 16 - first;
#pragma unroll
            for (int q = 0; q < 8; ++q) off[q] = (uint32_t)((16 * q + (lane >> 2)) * ld + m);
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                int64_t r = 8 * q + (lane >> 3);
                const int chunk = (lane & 7) ^ ((r >> 1) & 7);
                r = first + r < limit ? r : limit - 1 - first;
                off[q] = (uint32_t)(r * ld) + chunk * 16;
            }
        }
    };
    uint32_t oa[8], ob[8];
    lane_offsets(ATN, row0, p.rows, p.lda, oa);
    lane_offsets(BTN, col0, p.cols, p.ldb, ob);
    uint8_t *ring = lds + wave * WAVE_LDS;
    const uint32_t ring0 = lds_address(ring);
    auto issue = [&](int j) {  // stage j of this wave into buffer j % 2: QA + QB loads
        const uint8_t *ak = a_tile + (int64_t)(4 * j) * a_kstep;
        const uint8_t *bk = b_tile + (int64_t)(4 * j) * b_kstep;
        const uint32_t sa = ring0 + (j & 1) * STAGE;
#pragma unroll
        for (int q = 0; q < QA; ++q) dma16(ak, oa[q], sa + q * 1024);
#pragma unroll
        for (int q = 0; q < QB; ++q) dma16(bk, ob[q], sa + SLAB_A + q * 1024);
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    const int frow = lane & 31, fkb = lane >> 5, t16 = lane & 15;
    // fragment f (0, 1: a tile rows 32f ..; 2, 3: b) of half stage `sub` from buffer `s`: lane l
    // supplies tile row 32f + l%32 and contraction indices 64*sub + 32*(l/32) .. +31 -- two
    // 16-byte reads of a row-major slab, four transposing reads of eight contraction indices
    // each of a contraction-major one (see the general kernel)
    auto fragment = [&](const uint8_t *s, int sub, int f) -> i32x8 {
        const uint8_t *slab = s + (f >> 1) * SLAB_A;
        if ((f < 2 && ATN) || (f >= 2 && BTN)) {
            const int m = (f & 1) * 32 + (frow & 16);
            const int mc = m >> 4;
            i32x2 part[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = 64 * sub + 32 * fkb + 8 * e + (t16 >> 1);
                const int off = k * 64 + ((mc ^ (((k >> 2) & 1) << 1)) << 4) + 8 * (t16 & 1);
                part[e] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                    (__attribute__((address_space(3))) i32x2 *)(slab + off));
            }
            return i32x8{part[0].x, part[0].y, part[1].x, part[1].y, part[2].x, part[2].y, part[3].x, part[3].y};
        } else {
            const int row = (f & 1) * 32 + frow;
            const uint8_t *rp = slab + row * BK;
            const int sw = (row >> 1) & 7;
            const i32x4 h0 = *reinterpret_cast<const i32x4 *>(rp + (((4 * sub + 2 * fkb) ^ sw) << 4));
            const i32x4 h1 = *reinterpret_cast<const i32x4 *>(rp + (((4 * sub + 2 * fkb + 1) ^ sw) << 4));
            return __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };

    // (Issuing the fragment reads of a half stage ahead of the MFMAs of the one before it, as
    // the general kernel does, was measured and gained nothing here: the loop waits for loads.)
    if (mine > 0) issue(0);
    if (mine > 1) issue(1);
    for (int j = 0; j < mine; ++j) {
        if (j + 1 < mine) wait_vm_lds<QA + QB>();  // the loads of the next stage may fly
        else wait_vm_lds<0>();
        const uint8_t *s = ring + (j & 1) * STAGE;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            i32x8 af[MI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = fragment(s, sub, i);
            i32x8 bf[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) bf[j] = fragment(s, sub, 2 + j);
            // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets consecutive output columns
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf[j], af[i], acc[i][j], 1, 1, 0, 0, 0, 0);
        }
        if (j + 2 < mine) {
            // the loads below are invisible to the compiler (it could sink the multiplications
            // and their wait below them): wait for this wave's LDS reads explicitly
            wait_vm_lds<63>();
            issue(j + 2);
        }
    }
    wait_vm_lds<0>();

    // The four tiles meet in LDS: acc[i][j][4g + e] is row 32i + lane%32, column
    // 32j + 8g + 4*(lane/32) + e of this wave's tile.
    __syncthreads();  // every wave is done with its ring
    float *red = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                *reinterpret_cast<f32x4 *>(red + (wave * BM + 32 * i + frow) * RED_LD + 32 * j + 8 * g + 4 * fkb) = o;
            }
    __syncthreads();
    StatsAcc st;
    const bool fast_cols = (p.cols & 15) == 0;
    if (BM * BN == 64 * 64 || threadIdx.x < BM * BN / 16) {  // whole waves either way
        constexpr int CG = BN / 16;
        const int rr = threadIdx.x / CG, cg = threadIdx.x % CG;
        const int64_t r = row0 + rr, c = col0 + 16 * cg;
        float v[16];
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(red + (w * BM + rr) * RED_LD + 16 * cg + 4 * q);
                if (w == 0) {
                    v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
                } else {
                    v[4 * q] += x.x; v[4 * q + 1] += x.y; v[4 * q + 2] += x.z; v[4 * q + 3] += x.w;
                }
            }
        if (r < p.rows && c < p.cols) emit16<EPI>(p, split, r, c, v, st, fast_cols);
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
}

}  // namespace mp8
