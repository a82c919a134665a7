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
// done -- as a memory barrier for the compiler too: the kernel below mixes loads the compiler
// sees with direct-to-LDS loads it does not, and the count is only right if none of the former
// moves across the wait.
template <int n>
__device__ __forceinline__ void wait_vm_lds_fence() {
    static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(n) : "memory");
}

// y8[M, N] = Q(alpha * Q(x * scale)[M, K] . w8[K, N]) for N <= 128, writing Q(x * scale) as well.
// With one column tile the activations are read exactly once by the GEMM, so the kernel that
// rounds them can be the GEMM itself: a workgroup owns 64 rows; per 128-element stage of the
// contraction its threads load 64 x 128 FP32 (16-byte loads, a wave's load covering 512
// contiguous bytes of two rows; prefetched two stages ahead in registers), round each four to
// one dword of codes, store those to the 8-bit copy in
// HBM and into the row-major slab image of the MFMA kernels in LDS; the weights' stage
// (128 contraction rows x 128 columns, contraction-major) arrives by direct loads one stage
// ahead and is read with the transposing LDS reads.  The matrix work is negligible (the kernel
// moves 5 bytes per activation); what matters is the number of FP32 bytes in flight, hence the
// deep register prefetch and two workgroups per CU.
//
// Wave w: rows 32 * (w & 1) .., columns 64 * (w >> 1) .. of the tile.
// Everything a stage needs is requested two iterations before it is used: with the memory system
// saturated a request waits behind all the bytes in flight, so a load issued one iteration ahead
// would make every iteration last one such latency and leave half of the bytes in flight useless.
// Vector-memory counter per iteration i, in issue order after the barrier: 4 direct loads of the
// weights of stage i+2, 8 stores of the codes of stage i (fewer in a workgroup with rows beyond
// the matrix), 8 loads of the activations of stage i+2.  At the top of iteration i+1 the weights
// and activations of stage i+1, requested in iteration i-1, must have landed; operations
// complete in issue order, so "at most 20 outstanding" (12 where the number of stores is not
// known) implies that.
//
// QPLAIN: the activations are rounded to nearest even without saturation or statistics (the
// common case, kept free of the other cases' code).
template <int EPI, bool QPLAIN>
__global__ __launch_bounds__(256, 2) void gemm_qfwd_kernel(const GemmArgs p, const QuantArgs q) {
    constexpr int BM = 64, A_STAGE = BM * BK, B_SLAB = BK * 64, B_STAGE = 2 * B_SLAB;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[2 * A_STAGE + 3 * B_STAGE];
    uint8_t *lds_a = lds, *lds_b = lds + 2 * A_STAGE;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave & 1, wc = wave >> 1;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int ksteps = p.ksteps;
    const int64_t kc = (int64_t)ksteps * BK;

    // activations: item u (0..7) of a thread is four elements (one 16-byte load, one dword of
    // codes) of tile row 8u + t/32; a wave's load covers two rows of 512 contiguous bytes
    const int trow = threadIdx.x >> 5, c4 = threadIdx.x & 31;
    const float *src[8];
    uint8_t *dst[8];
    bool valid[8];
    uint32_t a_slot[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int row = 8 * u + trow;
        valid[u] = row0 + row < p.rows;
        const int64_t rr = valid[u] ? row0 + row : p.rows - 1;  // clamped rows are never stored
        src[u] = q.x + rr * kc + 4 * c4;
        dst[u] = q.x8 + rr * kc + 4 * c4;
        a_slot[u] = (uint32_t)(row * BK + ((((c4 >> 2) ^ ((row >> 1) & 7))) << 4) + 4 * (c4 & 3));
    }
    // weights: wave w brings contraction rows 64 * (w & 1) .. + 63 of the 64-column slab w >> 1;
    // a load covers 16 contraction rows of 64 bytes, lane l lands at (row l/4, slot l%4) and
    // fetches the chunk that belongs there under the swizzle of the narrow slabs
    const uint8_t *b_base = uniform_ptr(p.b);
    uint32_t ob[4];
    {
        const int chunk = (lane & 3) ^ (((lane >> 4) & 1) << 1);
        int64_t m = 64 * (wave >> 1) + 16 * chunk;
        m = m + 16 <= p.cols ? m : p.cols - 16;  // columns beyond the matrix: never stored
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
            ob[qq] = (uint32_t)((16 * (4 * (wave & 1) + qq) + (lane >> 2)) * p.ldb + m);
    }
    const uint32_t lds_b0 = lds_address(lds_b) + (wave >> 1) * B_SLAB + 4 * (wave & 1) * 1024;
    auto issue_b = [&](int ks, int ring) {  // stage ks into ring slot `ring` (= ks % 3)
        const uint8_t *bk = b_base + (int64_t)ks * BK * p.ldb;
        const uint32_t s = lds_b0 + ring * B_STAGE;
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) dma16(bk, ob[qq], s + qq * 1024);
    };

    f32x4 f[2][8];
    auto issue_x = [&](auto par, int ks) {
        constexpr int P = decltype(par)::value;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            f[P][u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src[u] + (int64_t)ks * BK));
    };

    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    const int frow = lane & 31, fkb = lane >> 5, t16 = lane & 15;
    const int fsw = (frow >> 1) & 7;
    const Philox rng(q.seed, q.offset);
    StatsAcc stx;
    const bool x_stats = q.stats != nullptr;

    const bool full = row0 + BM <= p.rows;  // every thread stores its codes: eight stores per stage
    issue_b(0, 0);
    issue_x(std::integral_constant<int, 0>{}, 0);
    if (ksteps > 1) {
        issue_b(1, 1);
        issue_x(std::integral_constant<int, 1>{}, 1);
    }
    int ring = 0;  // ring slot of the weights of the current stage

    auto stage = [&](auto par, int ks) {
        constexpr int P = decltype(par)::value;
        const bool counted_stores = ks > 0 && full;
        if (ks + 1 < ksteps) {
            if (counted_stores) wait_vm_lds_fence<20>();
            else wait_vm_lds_fence<12>();
        } else {
            if (counted_stores) wait_vm_lds_fence<8>();
            else wait_vm_lds_fence<0>();
        }
        // round this stage's activations; park the codes in registers
        uint32_t codes[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float y[4] = {f[P][u].x * q.scale, f[P][u].y * q.scale, f[P][u].z * q.scale, f[P][u].w * q.scale};
            if constexpr (QPLAIN) {
                codes[u] = e5m2_pack4<false>(y, 0u, 0u, false);
            } else {
                uint32_t r01 = 0, r23 = 0;
                if (q.sr) {
                    // elements e0 .. e0+3 of the tensor's row-major stream: halfwords e0 % 8 .. of
                    // Philox block e0 / 8
                    const int64_t e0 = (row0 + 8 * u + trow) * kc + (int64_t)ks * BK + 4 * c4;
                    const uint4 w = rng.block((uint64_t)e0 >> 3);
                    r01 = (e0 & 4) ? w.z : w.x;
                    r23 = (e0 & 4) ? w.w : w.y;
                }
                codes[u] = e5m2_pack4_rt(y, r01, r23, q.sr != 0, q.sat != 0);
                if (x_stats && valid[u]) stx.add4(y, codes[u]);
            }
        }
        uint8_t *sa = lds_a + (ks & 1) * A_STAGE;
#pragma unroll
        for (int u = 0; u < 8; ++u) *reinterpret_cast<uint32_t *>(sa + a_slot[u]) = codes[u];
        __syncthreads();  // codes of this stage visible; everyone is done reading stage ks - 1
        const int ring2 = ring == 0 ? 2 : ring - 1;  // (ks + 2) % 3: the slot stage ks - 1 used
        if (ks + 2 < ksteps) issue_b(ks + 2, ring2);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (valid[u]) *reinterpret_cast<uint32_t *>(dst[u] + (int64_t)ks * BK) = codes[u];
        if (ks + 2 < ksteps) issue_x(par, ks + 2);
        // matrix work of this stage
        const uint8_t *sb = lds_b + ring * B_STAGE + wc * B_SLAB;
        ring = ring == 2 ? 0 : ring + 1;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const uint8_t *ar = sa + (32 * wr + frow) * BK;
            const i32x4 a0 = *reinterpret_cast<const i32x4 *>(ar + (((4 * sub + 2 * fkb) ^ fsw) << 4));
            const i32x4 a1 = *reinterpret_cast<const i32x4 *>(ar + (((4 * sub + 2 * fkb + 1) ^ fsw) << 4));
            const i32x8 av = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
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
                const i32x8 bv = {part[0].x, part[0].y, part[1].x, part[1].y,
                                  part[2].x, part[2].y, part[3].x, part[3].y};
                // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets consecutive output columns
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv, av, acc[j], 1, 1, 0, 0, 0, 0);
            }
        }
    };
    for (int ks = 0; ks < ksteps; ks += 2) {
        stage(std::integral_constant<int, 0>{}, ks);
        if (ks + 1 < ksteps) stage(std::integral_constant<int, 1>{}, ks + 1);
    }

    // acc[j][4g + e]: row 32 wr + lane%32, column 64 wc + 32 j + 8g + 4 (lane/32) + e; one
    // exchange between the wave's halves leaves lane (row, h) with columns 16h .. 16h+15 of tile j
    StatsAcc st;
    const bool fast_cols = (p.cols & 15) == 0;
    const int64_t r = row0 + 32 * wr + frow;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        float v[16];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const auto sw = __builtin_amdgcn_permlane32_swap(f2u(acc[j][4 * g + e]),
                                                                 f2u(acc[j][4 * (g + 2) + e]), false, false);
                v[8 * g + e] = u2f(sw[0]);
                v[8 * g + 4 + e] = u2f(sw[1]);
            }
        const int64_t c = 64 * wc + 32 * j + 16 * fkb;
        if (r < p.rows && c < p.cols) emit16<EPI>(p, 0, r, c, v, st, fast_cols);
    }
    if constexpr (!QPLAIN) {
        if (x_stats) {
            stx.flush(q.stats);
            __syncthreads();  // the two reductions share their LDS words
        }
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
}

}  // namespace mp8
