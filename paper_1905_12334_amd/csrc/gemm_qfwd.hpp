// Forward GEMM that quantises its own activation operand: the Q node on the activations and
// the GEMM it feeds (Figure 1a of arXiv 1905.12334) as one kernel.
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

// The FP32 operand of a fused quantise-and-multiply kernel and its 8-bit copy.
struct QuantArgs {
    const float *x;   // [rows, contraction], dense
    uint8_t *x8;      // the rounded copy, same shape (the weight gradient reads it later)
    float scale;
    int sr, sat;
    uint64_t seed, offset;
    mp8_stats *stats;  // of x * scale and its codes, or null
};

// Wait until at most n vector-memory operations are outstanding and every LDS operation is
// done -- as a memory barrier for the compiler too.
template <int n>
__device__ __forceinline__ void wait_vm_lds_fence() {
    static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(n) : "memory");
}

// y8[M, N] = Q(alpha * Q(x * scale)[M, K] . w8[K, N]) for N <= 128, writing Q(x * scale) as well.
// With one column tile the activations are read exactly once by the GEMM, so the kernel that
// rounds them can be the GEMM itself.  A workgroup owns 64 (or 128) rows and has eight (twelve) waves in two roles:
//
//   the first four (eight) waves, the readers: per 128-element stage of the contraction they load 64 x 128 FP32
//     (16-byte loads, a wave's load covering 512 contiguous bytes of two rows, two or three
//     stages in flight in registers), round each four to one dword of codes and put the codes into the
//     row-major slab image of the MFMA kernels in LDS.  Their vector-memory queue holds nothing
//     but these loads: the kernel moves 5 bytes per activation and 4 of them come through here.
//   the last four waves, the multipliers: one stage behind, they bring the weights' stage (128 contraction
//     rows x 128 columns, contraction-major, direct loads two stages ahead into a ring of three),
//     multiply (multiplier v: rows (BM/2) (v & 1) .., columns 64 (v >> 1) .. of the tile, transposing
//     LDS reads for the weights), and copy the stage's codes from LDS to the 8-bit tensor in HBM
//     as whole 128-byte lines.
//
// What the split buys is bookkeeping, not time (a version with four waves that did everything
// took the same 32 us at 64 rows): a wave's memory operations complete in issue order, and with
// activation loads (which the compiler sees and places waits for), direct loads (which it does
// not) and stores in one queue, neither its counts nor hand-written ones stay simple.  Here the
// readers' queue holds nothing but loads the compiler knows, and only the multipliers count by
// hand; and the codes leave as whole lines instead of dwords.
//
// One barrier per iteration; iteration i: readers produce stage i, multipliers consume stage
// i - 1 (ksteps + 1 iterations).  Rows beyond the matrix are clamped to its last row in every
// respect (source, random stream, destination): their threads recompute and rewrite that row's
// codes, which keeps the number of memory operations per stage the same for every wave.
// Multiplier's queue per iteration, in issue order: 4 direct loads (stage s + 2, while there is
// one), BM/32 stores (stage s); before the barrier it waits for the direct loads of stage s + 1,
// after which only the younger operations (stores, 4 loads, stores) may be outstanding.
//
// QPLAIN: the activations are rounded to nearest even without saturation or statistics (the
// common case, kept free of the other cases' code).
//
// BM = 64 or 128 rows per workgroup (4 or 8 reading waves, always 4 multiplying waves).  Every
// workgroup passes over all of the weights once, and all workgroups want the same stage of them
// at the same time; with 128 rows that traffic through the L2 halves (measured 3 us of the 32
// at 64 rows), at the price of only ceil(M / 128) workgroups.
template <int EPI, bool QPLAIN, int BM>
__global__ __launch_bounds__(4 * BM + 256, BM == 64 ? 2 : 1) void gemm_qfwd_kernel(const GemmArgs p,
                                                                                  const QuantArgs q) {
    static_assert(BM == 64 || BM == 128, "rows per workgroup");
    constexpr int READERS = 4 * BM;   // threads that read; 256 more multiply
    constexpr int RB = BM / 64;       // 32-row blocks per multiplying wave
    // stages of activations in flight: three where the registers allow it (768 threads, lean rounding)
    constexpr int DEPTH = (BM == 128 && QPLAIN) ? 3 : 2;
    constexpr int A_STAGE = BM * BK, B_SLAB = BK * 64, B_STAGE = 2 * B_SLAB;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[2 * A_STAGE + 3 * B_STAGE];
    uint8_t *lds_a = lds, *lds_b = lds + 2 * A_STAGE;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int ksteps = p.ksteps;
    const int64_t kc = (int64_t)ksteps * BK;
    StatsAcc stx, st;

    if (wave < READERS / 64) {
        // ---- readers: item u (0..7) of a thread is four elements (one 16-byte load, one dword of
        // codes) of tile row (BM / 8) u + t/32
        const int trow = threadIdx.x >> 5, c4 = threadIdx.x & 31;
        const float *src[8];
        bool valid[8];
        uint32_t a_slot[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int row = (BM / 8) * u + trow;
            valid[u] = row0 + row < p.rows;
            const int64_t rr = valid[u] ? row0 + row : p.rows - 1;
            src[u] = q.x + rr * kc + 4 * c4;
            a_slot[u] = (uint32_t)(row * BK + ((((c4 >> 2) ^ ((row >> 1) & 7))) << 4) + 4 * (c4 & 3));
        }
        const Philox rng(q.seed, q.offset);
        const bool x_stats = q.stats != nullptr;
        f32x4 f[DEPTH][8];
        // Stages beyond the last one are "loaded" too (the first 16 bytes of x in every lane): the
        // number of loads in flight is then the same in every iteration, and the compiler's
        // placement of the waits for them stays exact across the loop.
        auto issue_x = [&](auto par, int ks) {
            constexpr int P = decltype(par)::value;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float *s = ks < ksteps ? src[u] + (int64_t)ks * BK : q.x;
                f[P][u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(s));
            }
        };
        auto stage = [&](auto par, int ks) {
            constexpr int P = decltype(par)::value;
            uint32_t codes[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float y[4] = {f[P][u].x * q.scale, f[P][u].y * q.scale, f[P][u].z * q.scale, f[P][u].w * q.scale};
                if constexpr (QPLAIN) {
                    codes[u] = e5m2_pack4<false, false>(y, 0u, 0u, false);
                } else {
                    uint32_t r01 = 0, r23 = 0;
                    if (q.sr) {
                        // elements e0 .. e0+3 of the tensor's row-major stream: halfwords e0 % 8 ..
                        // of Philox block e0 / 8
                        const int64_t e0 = (src[u] - q.x) + (int64_t)ks * BK;
                        const uint4 w = rng.block((uint64_t)e0 >> 3);
                        r01 = (e0 & 4) ? w.z : w.x;
                        r23 = (e0 & 4) ? w.w : w.y;
                    }
                    codes[u] = e5m2_pack4_rt<false>(y, r01, r23, q.sr != 0, q.sat != 0);
                    if (x_stats && valid[u]) stx.add4(y, codes[u]);
                }
            }
            issue_x(par, ks + DEPTH);
            uint8_t *sa = lds_a + (ks & 1) * A_STAGE;
#pragma unroll
            for (int u = 0; u < 8; ++u) *reinterpret_cast<uint32_t *>(sa + a_slot[u]) = codes[u];
            __syncthreads();  // stage ks is in LDS; the multipliers are done with stage ks - 2
        };
        // (the empty statements keep the two batches in this order: the compiler's bookkeeping of
        // loads in flight at the head of the loop is exact only if the way into the loop and the
        // way around it leave the same picture)
        const std::integral_constant<int, 0> c0{};
        const std::integral_constant<int, 1> c1{};
        issue_x(c0, 0);
        asm volatile("" ::: "memory");
        issue_x(c1, 1);
        asm volatile("" ::: "memory");
        int ks = 0;
        if constexpr (DEPTH == 2) {
            for (; ks + 1 < ksteps; ks += 2) {  // whole groups of stages: no way out of the middle
                stage(c0, ks);
                stage(c1, ks + 1);
            }
            if (ks < ksteps) stage(c0, ks);
        } else {
            const std::integral_constant<int, 2> c2{};
            issue_x(c2, 2);
            asm volatile("" ::: "memory");
            for (; ks + 2 < ksteps; ks += 3) {
                stage(c0, ks);
                stage(c1, ks + 1);
                stage(c2, ks + 2);
            }
            if (ks < ksteps) {
                stage(c0, ks);
                if (ks + 1 < ksteps) stage(c1, ks + 1);
            }
        }
        __syncthreads();  // the multipliers' last iteration
    } else {
        // ---- multipliers
        const int v = wave - READERS / 64, wr = v & 1, wc = v >> 1;
        // weights: wave v brings contraction rows 64 (v & 1) .. + 63 of the 64-column slab v >> 1;
        // a load covers 16 contraction rows of 64 bytes, lane l lands at (row l/4, slot l%4) and
        // fetches the chunk that belongs there under the swizzle of the narrow slabs
        const uint8_t *b_base = uniform_ptr(p.b);
        uint32_t ob[4];
        {
            const int chunk = (lane & 3) ^ (((lane >> 4) & 1) << 1);
            int64_t m = 64 * (v >> 1) + 16 * chunk;
            m = m + 16 <= p.cols ? m : p.cols - 16;  // columns beyond the matrix: never stored
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                ob[qq] = (uint32_t)((16 * (4 * (v & 1) + qq) + (lane >> 2)) * p.ldb + m);
        }
        const uint32_t lds_b0 = lds_address(lds_b) + (v >> 1) * B_SLAB + 4 * (v & 1) * 1024;
        // stage ks into ring slot `ring` (= ks % 3); nothing beyond the last stage
        auto issue_b = [&](int ks, int ring) {
            if (ks >= ksteps) return;
            const uint8_t *bk = b_base + (int64_t)ks * BK * p.ldb;
            const uint32_t s = lds_b0 + ring * B_STAGE;
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) dma16(bk, ob[qq], s + qq * 1024);
        };
        // the codes of a stage go to HBM as 16-byte pieces: piece q of tile row r sits in slot
        // q ^ ((r >> 1) & 7) of the slab; eight lanes store one 128-byte line
        constexpr int PIECES = BM / 32;  // per thread and stage
        const int ct = threadIdx.x - READERS;
        uint32_t piece_lds[PIECES];
        uint8_t *piece_dst[PIECES];
#pragma unroll
        for (int h = 0; h < PIECES; ++h) {
            const int pi = ct + 256 * h, row = pi >> 3, qq = pi & 7;
            const int64_t rr = row0 + row < p.rows ? row0 + row : p.rows - 1;
            piece_lds[h] = (uint32_t)(row * BK + ((qq ^ ((row >> 1) & 7)) << 4));
            piece_dst[h] = q.x8 + rr * kc + 16 * qq;
        }

        f32x16 acc[RB][2];
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
        const int frow = lane & 31, fkb = lane >> 5, t16 = lane & 15;
        const int fsw = (frow >> 1) & 7;

        issue_b(0, 0);
        issue_b(1, 1);
        if (ksteps > 1) wait_vm_lds_fence<4>();  // stage 0 of the weights (this wave's part)
        else wait_vm_lds_fence<0>();
        __syncthreads();         // iteration 0: the readers produce stage 0
        int ring = 0;            // ring slot of the weights of the current stage
        for (int s = 0; s < ksteps; ++s) {
            issue_b(s + 2, ring == 0 ? 2 : ring - 1);  // the slot stage s - 1 used
            const uint8_t *sa = lds_a + (s & 1) * A_STAGE;
            const uint8_t *sb = lds_b + ring * B_STAGE + wc * B_SLAB;
            ring = ring == 2 ? 0 : ring + 1;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                i32x8 bv[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int mc = (32 * j + (frow & 16)) >> 4;
                    i32x2 part[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int k = 64 * sub + 32 * fkb + 8 * e + (t16 >> 1);
                        const int off = k * 64 + ((mc ^ (((k >> 2) & 1) << 1)) << 4) + 8 * (t16 & 1);
                        part[e] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                            (__attribute__((address_space(3))) i32x2 *)(sb + off));
                    }
                    bv[j] = i32x8{part[0].x, part[0].y, part[1].x, part[1].y,
                                  part[2].x, part[2].y, part[3].x, part[3].y};
                }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const uint8_t *ar = sa + ((BM / 2) * wr + 32 * i + frow) * BK;
                    const i32x4 a0 = *reinterpret_cast<const i32x4 *>(ar + (((4 * sub + 2 * fkb) ^ fsw) << 4));
                    const i32x4 a1 = *reinterpret_cast<const i32x4 *>(ar + (((4 * sub + 2 * fkb + 1) ^ fsw) << 4));
                    const i32x8 av = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                    // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets consecutive output columns
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv[j], av, acc[i][j], 1, 1, 0, 0, 0, 0);
                }
            }
#pragma unroll
            for (int h = 0; h < PIECES; ++h) {
                const u32x4 o = *reinterpret_cast<const u32x4 *>(sa + piece_lds[h]);
                *reinterpret_cast<u32x4 *>(piece_dst[h] + (int64_t)s * BK) = o;
            }
            // this wave's part of stage s + 1 of the weights, requested one iteration ago (before the
            // loop for s = 0); younger: the stores of stage s - 1 (not for s = 0), 4 direct loads, the
            // stores of stage s
            if (s + 2 < ksteps) {
                if (s > 0) wait_vm_lds_fence<4 + 2 * PIECES>();
                else wait_vm_lds_fence<4 + PIECES>();
            } else {  // no direct loads were issued in this iteration
                if (s > 0) wait_vm_lds_fence<2 * PIECES>();
                else wait_vm_lds_fence<PIECES>();
            }
            __syncthreads();  // stage s + 1 of the codes and of the weights is complete
        }

        // acc[i][j][4g + e]: row (BM/2) wr + 32 i + lane%32, column 64 wc + 32 j + 8g + 4 (lane/32) + e;
        // one exchange between the wave's halves leaves lane (row, h) with columns 16h .. 16h+15
        const bool fast_cols = (p.cols & 15) == 0;
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            const int64_t r = row0 + (BM / 2) * wr + 32 * i + frow;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float vv[16];
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(f2u(acc[i][j][4 * g + e]),
                                                                         f2u(acc[i][j][4 * (g + 2) + e]), false, false);
                        vv[8 * g + e] = u2f(sw[0]);
                        vv[8 * g + 4 + e] = u2f(sw[1]);
                    }
                const int64_t c = 64 * wc + 32 * j + 16 * fkb;
                if (r < p.rows && c < p.cols) emit16<EPI>(p, 0, r, c, vv, st, fast_cols);
            }
        }
    }
    if constexpr (!QPLAIN) {
        if (q.stats != nullptr) {
            stx.flush(q.stats);
            __syncthreads();  // the two reductions share their LDS words
        }
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
}

}  // namespace mp8
