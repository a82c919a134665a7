// GEMM kernel for outputs with about one 128x128 tile per CU and a long contraction (the weight
// gradients of the Transformer layers): every wave multiplies the whole 128x128 tile, on its own
// quarter of the contraction, with no workgroup barrier in the loop.
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

// Why: with the general kernel a 128x128 tile gives each wave a 64x64 corner, i.e. eight MFMAs per
// 128-byte stage behind a workgroup barrier, and a stage costs a fixed 300-450 cycles of
// synchronisation (wait for the stage's loads, wait for the fragment reads just issued, the
// barrier itself) that only 512 cycles of matrix work stand against: the matrix cores are busy
// in little more than half of the cycles.  The 256x256 tile, with thirty-two MFMAs per wave and
// stage against the same fixed cost, keeps them busy in 0.87 -- but an output of 1024 x 4096 has
// only 64 such tiles for 256 CUs.
//
// Here a workgroup still owns one 128x128 tile, but the contraction is divided among its four
// waves (stage s of the workgroup's slice belongs to wave s % 4), and every wave computes the
// whole tile for its stages: sixteen accumulator tiles of 32x32 (all 256 accumulation registers),
// thirty-two MFMAs per stage, the instruction mix of a wave of the 256x256 kernel.  A wave shares
// nothing with the others until the end, so nothing in the loop waits for another wave:
//   - each wave has ONE stage buffer of its own (32 KB: 128 rows of a, 128 rows of b, 128 bytes of
//     contraction each), filled by its own direct-to-LDS loads and awaited with its own counter;
//   - when the stage has landed the wave reads ALL its fragments into registers (2 sub-steps x
//     8 fragments x 8 registers), which frees the buffer: the loads of the wave's next stage are
//     issued into it as soon as those reads have returned, one per MFMA slot, and have the rest
//     of the stage's MFMAs (about 1500 cycles) to arrive.
// At the end the four FP32 tiles meet in LDS, half a tile at a time, are added in wave order, and
// every thread owns sixteen consecutive columns of one row for the usual epilogues.
// Operand layouts and slab images as in the general kernel (ATN / BTN: contraction-major, through
// transposing LDS reads).
template <int EPI, bool ATN, bool BTN>
__global__ __launch_bounds__(256, 1) void gemm_wave128_kernel(const GemmArgs p) {
    static_assert(BTN || !ATN, "a alone contraction-major is not built");
    constexpr int BM = 128, BN = 128;
#ifndef MP8_W128_DMA_FROM
#define MP8_W128_DMA_FROM 8
#define MP8_W128_DMA_PER 2
#define MP8_W128_READ_LEAD 16
#endif
    constexpr int DMA_FROM = MP8_W128_DMA_FROM, DMA_PER = MP8_W128_DMA_PER;  // first slot with loads, loads per slot
    constexpr int READ_LEAD = MP8_W128_READ_LEAD;                            // fragments fetched ahead of the MFMAs
    static_assert(READ_LEAD >= 2 && 16 - READ_LEAD + 1 < DMA_FROM && DMA_FROM + 32 / DMA_PER <= 32, "slot schedule");
    constexpr int SLAB = 128 * BK;          // one operand's stage: 16 KB
    constexpr int WAVE_LDS = 2 * SLAB;      // a, then b
    constexpr int RED_LD = BN + 4;          // floats per row of a half tile parked for the reduction
    constexpr int RED_BYTES = 4 * 64 * RED_LD * 4;
    constexpr int LDS_BYTES = 4 * WAVE_LDS > RED_BYTES ? 4 * WAVE_LDS : RED_BYTES;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[LDS_BYTES];

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
    const uint8_t *a_tile = uniform_ptr((ATN ? p.a + row0 : p.a + row0 * p.lda) + (int64_t)(ks_begin + wave) * a_kstep);
    const uint8_t *b_tile = uniform_ptr((BTN ? p.b + col0 : p.b + col0 * p.ldb) + (int64_t)(ks_begin + wave) * b_kstep);
    // Direct loads, sixteen per operand and stage (1 KB each).  Row-major operand: load q brings
    // tile rows 8q .. 8q+7, lane i lands at (row i/8, slot i%8) and fetches chunk
    // (i%8) ^ ((row >> 1) & 7); rows beyond the matrix are clamped to its last row.
    // Contraction-major operand: load q brings contraction rows 8q .. 8q+7 of the 128 tile rows,
    // lane i lands at (row i/8, slot i%8) and fetches the chunk that the swizzle of those slabs
    // puts there, (i%8) ^ (2 * ((row >> 1) & 3)); chunks that would start beyond the matrix are
    // clamped to its last 16 rows.  (Clamped data is never stored.)
    auto lane_offsets = [&](bool km, int64_t first, int64_t limit, int64_t ld, uint32_t off[16]) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int r = 8 * q + (lane >> 3);
            if (km) {
                int64_t m = 16 * ((lane & 7) ^ (((r >> 1) & 3) << 1));
                m = first + m + 16 <= limit ? m : limit - 16 - first;
                off[q] = (uint32_t)(r * ld + m);
            } else {
                const int chunk = (lane & 7) ^ ((r >> 1) & 7);
                const int64_t rr = first + r < limit ? r : limit - 1 - first;
                off[q] = (uint32_t)(rr * ld) + chunk * 16;
            }
        }
    };
    uint32_t oa[16], ob[16];
    lane_offsets(ATN, row0, p.rows, p.lda, oa);
    lane_offsets(BTN, col0, p.cols, p.ldb, ob);
    uint8_t *buf = lds + wave * WAVE_LDS;
    const uint32_t buf0 = lds_address(buf);
    auto dma = [&](int j, int q) {  // load q (0 .. 31) of this wave's stage j
        if (q < 16) dma16(a_tile + (int64_t)(4 * j) * a_kstep, oa[q & 15], buf0 + q * 1024);
        else dma16(b_tile + (int64_t)(4 * j) * b_kstep, ob[q & 15], buf0 + SLAB + (q - 16) * 1024);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    const int frow = lane & 31, fkb = lane >> 5, t16 = lane & 15;
    // fragment f (0..3: a tile rows 32f ..; 4..7: b) of half stage `sub`: lane l supplies tile row
    // 32f + l%32 and contraction indices 64*sub + 32*(l/32) .. +31 -- two 16-byte reads of a
    // row-major slab, four transposing reads of eight contraction indices each of a
    // contraction-major one (see the general kernel)
    auto fragment = [&](int sub, int f) -> i32x8 {
        const uint8_t *slab = buf + (f >> 2) * SLAB;
        const int ff = f & 3;
        if ((f < 4 && ATN) || (f >= 4 && BTN)) {
            const int mc = (ff * 32 + (frow & 16)) >> 4;
            i32x2 part[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = 64 * sub + 32 * fkb + 8 * e + (t16 >> 1);
                const int off = k * 128 + ((mc ^ (((k >> 1) & 3) << 1)) << 4) + 8 * (t16 & 1);
                part[e] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) i32x2 *)(slab + off));
            }
            return i32x8{part[0].x, part[0].y, part[1].x, part[1].y, part[2].x, part[2].y, part[3].x, part[3].y};
        } else {
            const int row = ff * 32 + frow;
            const uint8_t *rp = slab + row * BK;
            const int sw = (row >> 1) & 7;
            const i32x4 h0 = *reinterpret_cast<const i32x4 *>(rp + (((4 * sub + 2 * fkb) ^ sw) << 4));
            const i32x4 h1 = *reinterpret_cast<const i32x4 *>(rp + (((4 * sub + 2 * fkb + 1) ^ sw) << 4));
            return __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };

    if (mine > 0) {
#pragma unroll
        for (int q = 0; q < 32; ++q) dma(0, q);
    }
    for (int j = 0; j < mine; ++j) {
        wait_vm_lds<0>();  // this wave's stage has landed (and nothing of its own is in flight in LDS)
        asm volatile("" ::: "memory");  // the fragment reads below stay below
        const bool more = j + 1 < mine;
        i32x8 fr[2][8];    // [half stage][fragment]
        // Fragments are fetched in the order in which the MFMAs first need them (per half stage:
        // b0, a0, b1, b2, b3, a1, a2, a3), the first four before the first MFMA, then one per MFMA
        // slot, READ_LEAD slots ahead of their first use: the wave starts multiplying as soon as
        // two fragments are there instead of after all thirty-two reads.
        auto read_frag = [&](int n) {  // n = 0 .. 15
            constexpr int order[8] = {4, 0, 5, 6, 7, 1, 2, 3};
            fr[n >> 3][order[n & 7]] = fragment(n >> 3, order[n & 7]);
        };
#pragma unroll
        for (int n = 0; n < READ_LEAD; ++n) read_frag(n);
        // Thirty-two MFMA slots.  MFMA m works on tile (i, jj) = (m / 4 % 4, m % 4) of half stage
        // m / 16, so a-fragments change slowly.  When the last fragment has returned (waited for
        // two slots after its read was issued) the buffer is free, and the loads of the wave's
        // next stage go out DMA_PER per slot.
#pragma unroll
        for (int m = 0; m < 32; ++m) {
            const int sub = m >> 4, i = (m >> 2) & 3, jj = m & 3;
            // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets consecutive output columns
            acc[i][jj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fr[sub][4 + jj], fr[sub][i], acc[i][jj], 1, 1, 0, 0, 0, 0);
            if (m + READ_LEAD < 16) read_frag(m + READ_LEAD);
            if (m == DMA_FROM - 1) {
                __builtin_amdgcn_sched_barrier(0);
                wait_vm_lds<63>();  // every fragment read of this stage has returned
            }
            if (m >= DMA_FROM && m < DMA_FROM + 32 / DMA_PER && more) {
#pragma unroll
                for (int d = 0; d < DMA_PER; ++d) dma(j + 1, DMA_PER * (m - DMA_FROM) + d);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vm_lds<0>();

    // The four tiles meet in LDS, 64 rows at a time: acc[i][j][4g + e] is row 32i + lane%32,
    // column 32j + 8g + 4*(lane/32) + e of this wave's tile.
    float *red = reinterpret_cast<float *>(lds);
    StatsAcc st;
    const bool fast_cols = (p.cols & 15) == 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        __syncthreads();  // every wave is done with its buffer / the previous half has been read
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x16 &t = acc[2 * h + ii][j];
                    f32x4 o = {t[4 * g], t[4 * g + 1], t[4 * g + 2], t[4 * g + 3]};
                    *reinterpret_cast<f32x4 *>(red + (wave * 64 + 32 * ii + frow) * RED_LD + 32 * j + 8 * g + 4 * fkb) = o;
                }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int item = threadIdx.x + 256 * it;  // 64 rows x 8 groups of sixteen columns
            const int rr = item >> 3, cg = item & 7;
            const int64_t r = row0 + 64 * h + rr, c = col0 + 16 * cg;
            float v[16];
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(red + (w * 64 + rr) * RED_LD + 16 * cg + 4 * q);
                    if (w == 0) {
                        v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
                    } else {
                        v[4 * q] += x.x; v[4 * q + 1] += x.y; v[4 * q + 2] += x.z; v[4 * q + 3] += x.w;
                    }
                }
            if (r < p.rows && c < p.cols) emit16<EPI>(p, split, r, c, v, st, fast_cols);
        }
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
}

}  // namespace mp8
