// GEMM kernel for contractions of one or two 128-byte stages.
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

// Short contraction (one or two 128-byte stages, both operands row-major).  Such a GEMM is all
// start-up and epilogue: every output byte costs only 128-256 bytes of MFMA input, so what
// bounds it is how many output lines are in flight.  This kernel is cut for that:
//   - one 128x128 tile per workgroup, all stages loaded at once (no ring, dynamic LDS of
//     32 KB per stage, so four workgroups fit a CU);
//   - wave w owns rows 32w .. 32w+31 and all 128 columns, so the wave writes whole 128-byte
//     lines of the 8-bit output;
//   - no LDS in the epilogue: the accumulator of a 32x32 tile has lane (row, h) hold columns
//     8g + 4h + e (g, e = 0..3); one v_permlane32_swap per register pair (g, g+2) leaves
//     lane (row, h) with the sixteen consecutive columns 16h .. 16h+15;
//   - tiles are numbered row-major, so a CU's consecutive tiles write neighbouring lines.
template <int EPI>
__global__ __launch_bounds__(256, EPI == EPI_FULL ? 4 : 5) void gemm_shortk_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds_dyn[];
    constexpr int BM = 128, BN = 128, A_BYTES = BM * BK, STAGE = (BM + BN) * BK;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // consecutive workgroup ids sit on different XCDs: give each XCD a contiguous tile range
    const uint32_t nb = gridDim.x, bid = blockIdx.x;
    const uint32_t xcd = bid & 7, per = nb >> 3, rem = nb & 7;
    const uint32_t pid = xcd * per + (xcd < rem ? xcd : rem) + (bid >> 3);
    uint32_t tn_;
    const int tm = __builtin_amdgcn_readfirstlane((int)fastdiv(pid, p.div_tn, tn_));
    const int tn = __builtin_amdgcn_readfirstlane((int)tn_);
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int ksteps = p.ksteps;  // 1 or 2

    // direct loads: same slab image as the main kernel (chunk c of row r in slot c ^ ((r>>1)&7))
    const int lrow = lane >> 3, lchunk = (lane & 7) ^ ((4 * wave + (lane >> 4)) & 7);
    const uint8_t *a_tile = uniform_ptr(p.a + row0 * p.lda);
    const uint8_t *b_tile = uniform_ptr(p.b + col0 * p.ldb);
    const uint32_t lds0 = lds_address(lds_dyn);
    uint32_t oa[4], ob[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int64_t r = 8 * (wave + 4 * q) + lrow, c = r;
        r = row0 + r < p.rows ? r : p.rows - 1 - row0;  // clamped rows are never stored
        c = col0 + c < p.cols ? c : p.cols - 1 - col0;
        oa[q] = (uint32_t)(r * p.lda) + lchunk * 16;
        ob[q] = (uint32_t)(c * p.ldb) + lchunk * 16;
    }
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        if (st < ksteps) {
            const uint32_t sa = lds0 + st * STAGE + wave * 1024;
#pragma unroll
            for (int q = 0; q < 4; ++q) dma16(a_tile + st * BK, oa[q], sa + q * 4096);
#pragma unroll
            for (int q = 0; q < 4; ++q) dma16(b_tile + st * BK, ob[q], sa + A_BYTES + q * 4096);
        }
    }

    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    const int frow = lane & 31, fkb = lane >> 5;
    const int fsw = (frow >> 1) & 7;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        if (st < ksteps) {
            if (st + 1 < ksteps) wait_vm_lds<8>();  // the eight loads of the next stage may fly
            else wait_vm_lds<0>();
            __syncthreads();
            const uint8_t *s = lds_dyn + st * STAGE;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int c0 = ((4 * sub + 2 * fkb) ^ fsw) * 16, c1 = ((4 * sub + 2 * fkb + 1) ^ fsw) * 16;
                const uint8_t *ar = s + (32 * wave + frow) * BK;
                const i32x4 a0 = *reinterpret_cast<const i32x4 *>(ar + c0);
                const i32x4 a1 = *reinterpret_cast<const i32x4 *>(ar + c1);
                const i32x8 av = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint8_t *br = s + A_BYTES + (32 * j + frow) * BK;
                    const i32x4 b0 = *reinterpret_cast<const i32x4 *>(br + c0);
                    const i32x4 b1 = *reinterpret_cast<const i32x4 *>(br + c1);
                    const i32x8 bv = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
                    // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets output columns
                    acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv, av, acc[j], 1, 1, 0, 0, 0, 0);
                }
            }
        }
    }

    const int64_t r = row0 + 32 * wave + frow;
    if constexpr (EPI == EPI_RNE) {
        // Codes first, then the exchange: four codes are one register, so a 32x32 tile needs two
        // swaps.  After swap(pk[g], pk[g+2]) the lower half holds its own columns 8g .. 8g+3
        // and the upper half's 8g+4 .. 8g+7; the upper half holds the lower half's
        // 16+8g .. 16+8g+3 and its own 16+8g+4 .. 16+8g+7: lane (row, h) has the 16-byte piece
        // 2j + h of its row.  The pieces then pass through the 4 KB of LDS that held this
        // wave's own rows of a (nobody else reads or writes them any more), so that eight
        // consecutive lanes store one whole 128-byte line: piece q of row rr sits in slot
        // q ^ ((rr >> 1) & 7), which keeps both the writes and the reads free of bank conflicts.
        uint8_t *mine = lds_dyn + 32 * wave * BK;
        auto tiles = [&](auto unit_alpha) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t pk[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float y[4] = {acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]};
                    if constexpr (!decltype(unit_alpha)::value) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) y[e] *= p.ep.alpha;
                    }
                    pk[g] = e5m2_pack4<false>(y, 0u, 0u, false);
                }
                const auto s0 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
                u32x4 o = {s0[0], s0[1], s1[0], s1[1]};
                *reinterpret_cast<u32x4 *>(mine + frow * BK + (((2 * j + fkb) ^ fsw) << 4)) = o;
            }
        };
        if (p.ep.alpha == 1.0f) tiles(std::true_type{});
        else tiles(std::false_type{});
        // the region is private to this wave: order its LDS writes before its reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int64_t c = col0 + 16 * (lane & 7);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int rr = 8 * k + (lane >> 3);
            const u32x4 o = *reinterpret_cast<const u32x4 *>(mine + rr * BK + (((lane & 7) ^ ((rr >> 1) & 7)) << 4));
            const int64_t ro = row0 + 32 * wave + rr;
            if (ro < p.rows && c < p.cols) *reinterpret_cast<u32x4 *>(p.ep.out8 + ro * p.cols + c) = o;
        }
        return;
    }
    StatsAcc stt;
    const bool fast_cols = (p.cols & 15) == 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v[16];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // lower half keeps its own columns 8g+e and receives the upper half's 8g+4+e;
                // the upper half receives the lower half's 8(g+2)+e and keeps its 8(g+2)+4+e
                const auto sw = __builtin_amdgcn_permlane32_swap(f2u(acc[j][4 * g + e]),
                                                                 f2u(acc[j][4 * (g + 2) + e]), false, false);
                v[8 * g + e] = u2f(sw[0]);
                v[8 * g + 4 + e] = u2f(sw[1]);
            }
        const int64_t c = col0 + 32 * j + 16 * fkb;
        if (r < p.rows && c < p.cols) emit16<EPI>(p, 0, r, c, v, stt, fast_cols);
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) stt.flush(p.ep.stats);
    }
}

}  // namespace mp8
