// What the GEMM kernels share: argument structs, the epilogue of one output run (one rounding
// of the complete FP32 sum, Section 3 of arXiv 1905.12334), the workgroup -> tile map, and the
// direct-to-LDS load with its hand-tracked wait.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <type_traits>

#include "mp8_device.hpp"

namespace mp8 {

using i32x8 = int __attribute__((ext_vector_type(8)));
using i32x4 = int __attribute__((ext_vector_type(4)));
using i32x2 = int __attribute__((ext_vector_type(2)));
using f32x16 = float __attribute__((ext_vector_type(16)));

constexpr int BK = 128;  // bytes (= elements) of contraction per pipeline stage

// Division of a 31-bit number by a fixed divisor with a precomputed reciprocal:
// m = floor(2^32 / d) (all ones for d = 1) makes mulhi(x, m) the quotient or one less.
struct FastDiv {
    uint32_t d, m;
};
static inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.m = d <= 1 ? 0xFFFFFFFFu : (uint32_t)((1ull << 32) / d);
    return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t x, const FastDiv &f, uint32_t &rem) {
    uint32_t q = __umulhi(x, f.m);
    rem = x - q * f.d;
    if (rem >= f.d) {
        ++q;
        rem -= f.d;
    }
    return q;
}

struct Epilogue {
    float alpha;
    float *acc;
    int acc_mode;
    uint8_t *out8;
    uint8_t *out8_t;
    int sr;
    int sat;
    uint64_t seed, offset;
    mp8_stats *stats;
    int want_codes;  // the caller consumes the returned codes even if nothing is stored
    int64_t rows, cols;
    // Convolution outputs live on the zero-padded pixel grid (rows = padded pixels): rows that
    // are padding receive zero codes and stay out of the statistics.  mask = 0: no masking.
    int mask;
    int hh;              // H + 2
    int64_t valid_rows;  // B * (H+2) * (W+2); rows beyond are padding as well
    FastDiv div_img;     // by (H+2) * (W+2)
    FastDiv div_w2;      // by W + 2
};

// Is output row r a padding pixel of the convolution grid?
__device__ __forceinline__ bool conv_padding_row(const Epilogue &ep, int64_t r) {
    if (r >= ep.valid_rows) return true;
    uint32_t rem, x;
    fastdiv((uint32_t)r, ep.div_img, rem);
    const uint32_t y = fastdiv(rem, ep.div_w2, x);
    return y == 0 || y == (uint32_t)ep.hh - 1 || x == 0 || x == ep.div_w2.d - 1;
}

// What a convolution adds to the operand addressing (conv = 0: plain GEMM).
struct ConvArgs {
    int w2;               // W + 2: a tap (r, s) shifts the pixel row by (r-1)*w2 + (s-1)
    FastDiv div_cpb;      // by units_per_tap
    int units_per_tap;    // 64-byte units of the contraction per tap (contracted channels / 64)
    int odd_units;        // the contraction has an odd number of units: its last stage starts one early
    int64_t b_tap_stride; // backward data: bytes between the weight slabs of two taps
    FastDiv div_ci;       // weight gradient: by Cin (tile row -> tap, first channel)
};

struct GemmArgs {
    const uint8_t *a;
    const uint8_t *b;
    int64_t lda, ldb;
    int64_t rows, cols;
    int ksteps;         // contraction length / BK (pipeline stages)
    int splits;         // number of contraction slices
    int tiles_m, tiles_n;
    // host-side precomputation for the workgroup -> (slice, tile) map, so that the kernel's
    // start-up does no integer division
    FastDiv div_tiles;  // by tiles_m * tiles_n
    FastDiv div_band;   // by 8 * tiles_n
    FastDiv div_tail;   // by the height of the last band of tile rows (tiles_m % 8, or 8)
    FastDiv div_tn;     // by tiles_n
    int ks_per, ks_extra;  // ksteps / splits and ksteps % splits
    float *partial;     // [splits, rows, cols] when splits > 1
    ConvArgs cv;
    Epilogue ep;
};

// One output element, any shape: optional FP32 accumulate / store, one rounding to 8 bits,
// optional transposed copy, statistics.  Only the finishing kernels use it (ragged shapes).
__device__ __forceinline__ uint32_t finish1(const Epilogue &ep, int64_t r, int64_t c, float v,
                                            StatsAcc &st) {
    const int64_t i = r * ep.cols + c;
    if (ep.acc_mode != 0) {
        if (ep.acc_mode == 2) v += ep.acc[i];
        ep.acc[i] = v;
    }
    if (ep.out8 == nullptr && ep.out8_t == nullptr && ep.stats == nullptr && !ep.want_codes) return 0;
    if (ep.mask && conv_padding_row(ep, r)) {
        if (ep.out8 != nullptr) ep.out8[i] = 0;
        if (ep.out8_t != nullptr) ep.out8_t[c * ep.rows + r] = 0;
        return 0;
    }
    const float y = v * ep.alpha;
    uint32_t code;
    if (ep.sr) {
        const Philox rng(ep.seed, ep.offset);
        uint32_t r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
        code = e5m2_from_f32_bits<true>(f2u(y), r16, ep.sat != 0);
    } else {
        code = e5m2_from_f32_bits<false>(f2u(y), 0u, ep.sat != 0);
    }
    if (ep.stats != nullptr) st.add1(y, code);
    if (ep.out8 != nullptr) ep.out8[i] = (uint8_t)code;
    if (ep.out8_t != nullptr) ep.out8_t[c * ep.rows + r] = (uint8_t)code;
    return code;
}

// Finish sixteen consecutive columns c .. c+15 (c % 16 == 0) of output row r of an output
// whose row length is a multiple of 16: 16-byte accesses, two Philox blocks, hardware
// conversions.  Written to stay small: the rounding mode is a run-time flag and the rare
// conversions are out of line.
__device__ __forceinline__ void finish16(const Epilogue &ep, int64_t r, int64_t c, float v[16],
                                         StatsAcc &st) {
    const int64_t i0 = r * ep.cols + c;
    if (ep.acc_mode != 0) {
        f32x4 *p = reinterpret_cast<f32x4 *>(ep.acc + i0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (ep.acc_mode == 2) {
                f32x4 o = p[q];
                v[4 * q] += o.x; v[4 * q + 1] += o.y; v[4 * q + 2] += o.z; v[4 * q + 3] += o.w;
            }
            f32x4 n = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
            p[q] = n;
        }
    }
    if (ep.out8 == nullptr && ep.out8_t == nullptr && ep.stats == nullptr) return;
    const bool padding = ep.mask && conv_padding_row(ep, r);
    uint32_t rw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (ep.sr) {
        const Philox rng(ep.seed, ep.offset);
        uint4 w0 = rng.block((uint64_t)i0 >> 3), w1 = rng.block(((uint64_t)i0 >> 3) + 1);
        rw[0] = w0.x; rw[1] = w0.y; rw[2] = w0.z; rw[3] = w0.w;
        rw[4] = w1.x; rw[5] = w1.y; rw[6] = w1.z; rw[7] = w1.w;
    }
    uint32_t pk[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float y[4] = {v[4 * q] * ep.alpha, v[4 * q + 1] * ep.alpha, v[4 * q + 2] * ep.alpha,
                      v[4 * q + 3] * ep.alpha};
        pk[q] = e5m2_pack4_rt(y, rw[2 * q], rw[2 * q + 1], ep.sr != 0, ep.sat != 0);
        if (padding) pk[q] = 0;
        else if (ep.stats != nullptr) st.add4(y, pk[q]);
    }
    if (ep.out8 != nullptr) {
        u32x4 o = {pk[0], pk[1], pk[2], pk[3]};
        *reinterpret_cast<u32x4 *>(ep.out8 + i0) = o;
    }
    if (ep.out8_t != nullptr) {
        uint8_t *t = ep.out8_t + c * ep.rows + r;
#pragma nounroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t w = q == 0 ? pk[0] : q == 1 ? pk[1] : q == 2 ? pk[2] : pk[3];
            t[(4 * q + 0) * ep.rows] = (uint8_t)w;
            t[(4 * q + 1) * ep.rows] = (uint8_t)(w >> 8);
            t[(4 * q + 2) * ep.rows] = (uint8_t)(w >> 16);
            t[(4 * q + 3) * ep.rows] = (uint8_t)(w >> 24);
        }
    }
}

// Map the linear workgroup id to (slice, tile row, tile column).  Consecutive ids go to
// different XCDs (round robin), so ids are first regrouped so that each XCD works on a
// contiguous range of tiles and its L2 sees operand reuse; inside the range, tiles are
// walked in bands of 8 tile-rows.
__device__ __forceinline__ void map_block(const GemmArgs &p, int &split, int &tm, int &tn) {
    const uint32_t nb = gridDim.x, bid = blockIdx.x;
    const uint32_t xcd = bid & 7, idx = bid >> 3;
    const uint32_t per = nb >> 3, rem = nb & 7;
    const uint32_t pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
    uint32_t t, in;
    split = (int)fastdiv(pid, p.div_tiles, t);
    constexpr uint32_t GM = 8;
    const uint32_t g = fastdiv(t, p.div_band, in);
    const uint32_t first = g * GM;
    if ((uint32_t)p.tiles_m - first >= GM) {
        tm = (int)(first + (in & (GM - 1)));
        tn = (int)(in >> 3);
    } else {
        uint32_t r;
        tn = (int)fastdiv(in, p.div_tail, r);
        tm = (int)(first + r);
    }
}

enum { EPI_PARTIAL = 0, EPI_RNE = 1, EPI_FULL = 2 };

// What a tile kernel does with sixteen consecutive columns c .. c+15 (c % 16 == 0) of output row
// r, per epilogue variant (described at the main kernel): FP32 to slice `split` of the workspace, the RNE-only
// conversion, or the complete epilogue.
template <int EPI>
__device__ __forceinline__ void emit16(const GemmArgs &p, int split, int64_t r, int64_t c,
                                       float v[16], StatsAcc &st, bool fast_cols) {
    if constexpr (EPI == EPI_PARTIAL) {
        float *dst = p.partial + ((int64_t)split * p.rows + r) * p.cols + c;
        if (fast_cols) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 o = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
                reinterpret_cast<f32x4 *>(dst)[q] = o;
            }
        } else {
            // constant indices only: a run-time index would move v out of the registers
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (c + e < p.cols) dst[e] = v[e];
        }
    } else if constexpr (EPI == EPI_RNE) {
        // the host sends only row lengths that are multiples of 16 here
        uint32_t pk[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float y[4] = {v[4 * q] * p.ep.alpha, v[4 * q + 1] * p.ep.alpha,
                          v[4 * q + 2] * p.ep.alpha, v[4 * q + 3] * p.ep.alpha};
            pk[q] = e5m2_pack4<false>(y, 0u, 0u, false);
        }
        if (p.ep.mask && conv_padding_row(p.ep, r)) pk[0] = pk[1] = pk[2] = pk[3] = 0;
        u32x4 o = {pk[0], pk[1], pk[2], pk[3]};
        *reinterpret_cast<u32x4 *>(p.ep.out8 + r * p.cols + c) = o;
    } else {
        finish16(p.ep, r, c, v, st);
    }
}

// Wait until at most n vector-memory operations of this wave are outstanding and all of its
// LDS operations have completed (gfx9 encoding: vmcnt in bits 3:0 and 15:14, lgkmcnt in
// bits 11:8, expcnt left at "no wait").
template <int n>
__device__ __forceinline__ void wait_vm_lds() {
    static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// One direct-to-LDS load: 64 lanes x 16 bytes land at LDS byte address lds_addr + lane * 16
// (lds_addr is wave-uniform and travels in M0).  Written as inline assembly on purpose: the
// compiler then neither knows nor tracks that this is a load into LDS, and would otherwise
// put a wait for ALL outstanding loads in front of every later LDS read, which serialises
// the prefetch ring.  Completion is tracked by hand with the vector-memory counter.
__device__ __forceinline__ void dma16(const uint8_t *gbase, uint32_t lane_off, uint32_t lds_addr) {
    // global address = wave-uniform base (SGPR pair) + per-lane 32-bit offset
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off), "s"(gbase), "s"(lds_addr)
                 : "memory", "m0");
}

// Tell the compiler that a pointer is the same in every lane (keeps it in scalar registers).
__device__ __forceinline__ const uint8_t *uniform_ptr(const uint8_t *p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const uint8_t *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)p;
}

}  // namespace mp8
