// mp8_gemm_fp8: the FP8 compute primitive of Section 3 (arXiv 1905.12334) for gfx950 --
// two 8-bit (1,5,2) operands, FP32 accumulation on the matrix cores, and the Q node of
// Figure 1a (one rounding of the complete FP32 sum to 8 bits, RNE or stochastic) fused into
// the epilogue.  The three training GEMMs (forward, backward-data, weight-gradient) are the
// same contraction  out[r,c] = sum_j a[r,j] * b[c,j]  on differently oriented operands.
//
// Main kernel: 256 threads (4 waves), block tile BM x BN, 128 bytes of contraction per
// pipeline stage.  Operand slabs travel HBM -> LDS with direct-to-LDS 16-byte loads into a
// ring of 2-4 stages (issued from inline asm with hand-tracked wait counts), are read as
// 32-byte-per-lane fragments into double-buffered registers and multiplied with
// v_mfma_f32_32x32x64_f8f6f4 in its bf8 x bf8 form.  The main loop is slot-scheduled: one
// MFMA per slot, with the LDS reads and direct loads of the next half-stage spread in its
// shadow.  The LDS image is XOR-swizzled in 16-byte chunks so that fragment reads are
// bank-conflict free; because direct-to-LDS writes are lane-contiguous the swizzle is applied
// to the global address each lane fetches.  The operands are fed to the MFMA swapped (b as
// the "row" matrix) so that each lane ends up with consecutive output columns of one row.
// The kernel is instantiated per epilogue variant (FP32 partial tile, RNE only, everything) to
// keep each instance's code small.
//
// Split contraction, FP32 / transposed outputs, ragged column counts: the main kernel writes
// FP32 tiles and a second kernel sums the slices in order and applies the epilogue -- the sum
// is rounded exactly once.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <type_traits>

#include "mp8_device.hpp"

namespace mp8 {

using i32x8 = int __attribute__((ext_vector_type(8)));
using i32x4 = int __attribute__((ext_vector_type(4)));
using i32x2 = int __attribute__((ext_vector_type(2)));
using f32x16 = float __attribute__((ext_vector_type(16)));

constexpr int BK = 128;  // bytes (= elements) of contraction per pipeline stage

#ifdef MP8_TRACE
// Diagnostic build only: cycle stamps of one block, [wave][stage][point].
#ifndef MP8_TRACE_BLOCK
#define MP8_TRACE_BLOCK 0
#endif
__device__ unsigned long long mp8_trace_buf[4][160][8];
#define MP8_STAMP(pt) do { if (blockIdx.x == MP8_TRACE_BLOCK && lane == 0 && t < 159) mp8_trace_buf[wave][t][pt] = __builtin_readcyclecounter(); } while (0)
#define MP8_STAMP_PHASE(pt) do { if (blockIdx.x == MP8_TRACE_BLOCK && (threadIdx.x & 63) == 0) mp8_trace_buf[threadIdx.x >> 6][159][pt] = __builtin_readcyclecounter(); } while (0)
// constant-rate (100 MHz) clock stamps of every workgroup: [block][point]
__device__ unsigned long long mp8_block_times[16384][4];
#define MP8_BLOCK_STAMP(pt) do { if (threadIdx.x == 0 && blockIdx.x < 16384) mp8_block_times[blockIdx.x][pt] = wall_clock64(); } while (0)
#else
#define MP8_BLOCK_STAMP(pt) do { } while (0)
#define MP8_STAMP(pt) do { } while (0)
#define MP8_STAMP_PHASE(pt) do { } while (0)
#endif

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
    FastDiv div_cpb;      // by the number of 128-byte stages per tap (channels / 128)
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
                 : "memory");
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

// Main kernel.  256 threads = WGM x WGN waves, block tile BM x BN, NSTAGE-deep ring of
// 128-byte-wide operand slabs in LDS (BK = 128: whole 128-byte lines travel from L2 to the
// CU exactly once).  One slab = two MFMA sub-steps of 64.
//
// Pipeline of stage t, per wave (one barrier per stage, placed in its middle):
//   sub-step 0:  read the fragments of (t, 1) into register set 1; multiply set 0 = (t, 0)
//   middle:      wait for this wave's loads of stage t+1 and for its LDS reads; barrier --
//                now stage t+1 is complete in LDS and nobody needs the buffer of stage t;
//                issue the direct-to-LDS loads of stage t+NSTAGE into that buffer
//   sub-step 1:  read the fragments of (t+1, 0) into set 0; multiply set 1 = (t, 1)
// A load therefore has NSTAGE-1 stages of MFMA work to arrive, fragment reads are always one
// sub-step ahead of their use, and the barrier is hidden behind queued MFMAs.
//
// LDS image of a slab: row r occupies 128 bytes, its 16-byte chunk c sits at slot
// c ^ ((r >> 1) & 7).  The LDS serves a 16-byte-per-lane read sixteen lanes at a time over
// its 64 banks (256 bytes = two rows); a fragment read has lanes 0..15 on rows r..r+15 with
// the same chunk, and with this swizzle the sixteen pieces fall into sixteen different
// 16-byte bank groups.  Direct-to-LDS writes are lane-contiguous, so the swizzle is applied
// to the global address each lane fetches.
// EPI selects what happens to the finished FP32 tile (one kernel per variant keeps each
// kernel's code, and with it the cold instruction-cache cost of every launch, small):
//   EPI_PARTIAL  FP32 tile to the workspace (split contraction, or options the fused
//                epilogue does not carry); the finishing kernel does the rest
//   EPI_RNE      out8 = Q_RNE(alpha * acc), nothing else
//   EPI_FULL     out8 with run-time rounding mode, saturation and statistics

// CONV: 0 plain GEMM; 1 / 2 / 3 forward / backward-data / weight-gradient 3x3 convolution on
// zero-padded channels-last tensors, where a tap of the filter is a shift of the pixel row:
//   1  a[r, (tap, ci)] = x[r + shift(tap), ci]      a plain, b = w [9 Cin, Cout] contraction-major
//   2  a[r, (tap, co)] = e[r - shift(tap), co]      a plain, b[ci, (tap, co)] = w[tap][ci][co]
//   3  a[(tap, ci), r] = x[r + shift(tap), ci]      both contraction-major, tap fixed per tile row
// so only the base address of a stage (1, 2) or of a tile (3) differs from the plain GEMM.
template <int BM, int BN, int WGM, int WGN, int NSTAGE, int MINBLOCKS, int EPI, bool ATN = false,
          bool BTN = false, int CONV = 0>
__global__ __launch_bounds__(256, MINBLOCKS) void gemm_mfma_kernel(const GemmArgs p) {
    static_assert(CONV == 0 || (CONV == 1 && !ATN && BTN) || (CONV == 2 && !ATN && !BTN) ||
                      (CONV == 3 && ATN && BTN), "operand layouts of the convolution forms");
    static_assert((!ATN || BM % 128 == 0 || BM == 64) && (!BTN || BN % 128 == 0 || BN == 64),
                  "contraction-major operands: panels of 128 (or one of 64) tile rows");
    static_assert(WGM * WGN == 4, "four waves");
    static_assert(NSTAGE >= 2, "ring depth");
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    constexpr int MT = WTM / 32, NT = WTN / 32;    // 32x32 MFMA tiles per wave
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    constexpr int A_DMA = BM / 32, B_DMA = BN / 32;  // direct loads per wave per stage
    constexpr int G = A_DMA + B_DMA;
    static_assert(G * (NSTAGE - 2) < 64, "vmcnt range");
    // the operand ring, reused by the epilogue for FP32 row bands (2 x 32 rows per wave)
    constexpr int EP_BYTES = 4 * (MT >= 2 ? 2 : 1) * 32 * (WTN + 4) * 4;
    constexpr int LDS_BYTES = NSTAGE * STAGE > EP_BYTES ? NSTAGE * STAGE : EP_BYTES;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[LDS_BYTES];

    MP8_STAMP_PHASE(0);
    MP8_BLOCK_STAMP(0);
    int split, tm, tn;
    map_block(p, split, tm, tn);
    split = __builtin_amdgcn_readfirstlane(split);
    tm = __builtin_amdgcn_readfirstlane(tm);
    tn = __builtin_amdgcn_readfirstlane(tn);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;

    // contraction slice of this workgroup, in stages of 128
    const int per = p.ks_per, extra = p.ks_extra;
    const int ks_begin = split * per + (split < extra ? split : extra);
    const int ks_count = __builtin_amdgcn_readfirstlane(per + (split < extra ? 1 : 0));

    // Direct loads.  Load q of this wave brings rows 8*(wave + 4q) .. +7 of the slab; lane i
    // lands at (row i/8, slot i%8) and therefore fetches global chunk (i%8) ^ ((row >> 1) & 7)
    // of that row; with row = 8*(wave + 4q) + i/8 that is ((4*wave + i/16) & 7).  Rows beyond
    // the matrix are clamped to its last row (never stored).  Addresses are a wave-uniform
    // base (tile origin + stage) plus a 32-bit lane offset.
    //
    // Contraction-major operands (ATN: a is [kc, rows]; BTN: b is [kc, cols]) use the same LDS
    // geometry with the roles swapped: a slab is cut into panels of 128 tile rows, each panel
    // is 128 contraction rows of 128 bytes, chunk c of contraction row k sits in slot
    // c ^ (2 * ((k >> 1) & 3)).  Chunks that would start beyond the matrix are clamped to its
    // last 16 rows (never stored).
    // A tile of only 64 rows is one panel of 128 contraction rows of 64 bytes: a direct load
    // then covers 16 contraction rows, lane i lands at (row i/4, slot i%4), and chunk c of
    // contraction row k sits in slot c ^ (2 * ((k >> 2) & 1)).
    // These two swizzles are cut for the transposing reads below, which the LDS serves 32 lanes
    // at a time: lanes 0..15 name contraction rows k0 .. k0+7 of one chunk, lanes 16..31 the
    // same rows of the next chunk.  Rows of equal parity (wide) or equal position within a
    // 256-byte bank period (narrow) fall on the same banks unless their slots differ, so the
    // rows' slots must differ in bit 1 or above (bit 0 tells the two chunks apart): the 32 lanes
    // then cover all 64 banks exactly once.  (With the fragment swizzle of the row-major slabs
    // half of the LDS cycles of these reads were bank conflicts.)
    const int lrow = lane >> 3, lchunk = (lane & 7) ^ ((4 * wave + (lane >> 4)) & 7);
    const int lchunk_t = (lane & 7) ^ (((lane >> 4) & 3) << 1);
    const int lrow64 = lane >> 2, lchunk64 = (lane & 3) ^ (((lane >> 4) & 1) << 1);
    const int64_t a_kstep = ATN ? (int64_t)BK * p.lda : BK, b_kstep = BTN ? (int64_t)BK * p.ldb : BK;
    auto tap_shift = [&](uint32_t tap) {  // pixel-row shift of filter tap (r, s) = (tap / 3, tap % 3)
        const int r = (int)((tap * 11u) >> 5);
        return (r - 1) * p.cv.w2 + ((int)tap - 3 * r - 1);
    };
    const uint8_t *a_origin, *b_origin;
    if constexpr (CONV == 1 || CONV == 2) {
        a_origin = p.a + row0 * p.lda;  // the stage's tap and channel part are added per stage
    } else if constexpr (CONV == 3) {
        uint32_t ci0;
        const uint32_t tap = fastdiv((uint32_t)row0, p.cv.div_ci, ci0);
        a_origin = p.a + (int64_t)tap_shift(tap) * p.lda + ci0 + (int64_t)ks_begin * a_kstep;
    } else {
        a_origin = ATN ? p.a + (int64_t)ks_begin * a_kstep + row0 : p.a + row0 * p.lda + (int64_t)ks_begin * BK;
    }
    if constexpr (CONV == 2) b_origin = p.b + col0 * p.ldb;
    else b_origin = BTN ? p.b + (int64_t)ks_begin * b_kstep + col0 : p.b + col0 * p.ldb + (int64_t)ks_begin * BK;
    const uint8_t *a_tile = uniform_ptr(a_origin);
    const uint8_t *b_tile = uniform_ptr(b_origin);
    // base addresses of stage `kstage` of this workgroup's slice
    auto a_stage = [&](int kstage) -> const uint8_t * {
        if constexpr (CONV == 1 || CONV == 2) {
            uint32_t part;
            const uint32_t tap = fastdiv((uint32_t)(ks_begin + kstage), p.cv.div_cpb, part);
            const int sh = CONV == 1 ? tap_shift(tap) : -tap_shift(tap);
            return a_tile + (int64_t)sh * p.lda + part * BK;
        } else {
            return a_tile + (int64_t)kstage * a_kstep;
        }
    };
    auto b_stage = [&](int kstage) -> const uint8_t * {
        if constexpr (CONV == 2) {
            uint32_t part;
            const uint32_t tap = fastdiv((uint32_t)(ks_begin + kstage), p.cv.div_cpb, part);
            return b_tile + (int64_t)tap * p.cv.b_tap_stride + part * BK;
        } else {
            return b_tile + (int64_t)kstage * b_kstep;
        }
    };
    uint32_t oa[A_DMA], ob[B_DMA];
#pragma unroll
    for (int q = 0; q < A_DMA; ++q) {
        if constexpr (ATN) {
            const int64_t krow = BM == 64 ? 16 * (wave + 4 * q) + lrow64 : 8 * (wave + 4 * (q & 3)) + lrow;
            int64_t m = BM == 64 ? 16 * lchunk64 : 128 * (q >> 2) + 16 * lchunk_t;
            m = row0 + m + 16 <= p.rows ? m : p.rows - 16 - row0;
            oa[q] = (uint32_t)(krow * p.lda + m);
        } else {
            int64_t r = 8 * (wave + 4 * q) + lrow;
            r = row0 + r < p.rows ? r : p.rows - 1 - row0;
            oa[q] = (uint32_t)(r * p.lda) + lchunk * 16;
        }
    }
#pragma unroll
    for (int q = 0; q < B_DMA; ++q) {
        if constexpr (BTN) {
            const int64_t krow = BN == 64 ? 16 * (wave + 4 * q) + lrow64 : 8 * (wave + 4 * (q & 3)) + lrow;
            int64_t m = BN == 64 ? 16 * lchunk64 : 128 * (q >> 2) + 16 * lchunk_t;
            m = col0 + m + 16 <= p.cols ? m : p.cols - 16 - col0;
            ob[q] = (uint32_t)(krow * p.ldb + m);
        } else {
            int64_t c = 8 * (wave + 4 * q) + lrow;
            c = col0 + c < p.cols ? c : p.cols - 1 - col0;
            ob[q] = (uint32_t)(c * p.ldb) + lchunk * 16;
        }
    }
    const uint32_t lds0 = lds_address(lds);
    auto issue_loads = [&](int kstage) {
        const uint32_t sa = lds0 + (kstage % NSTAGE) * STAGE + wave * 1024;
        const uint32_t sb = sa + A_BYTES;
        const uint8_t *ak = a_stage(kstage);
        const uint8_t *bk = b_stage(kstage);
#pragma unroll
        for (int q = 0; q < A_DMA; ++q) dma16(ak, oa[q], sa + q * 4096);
#pragma unroll
        for (int q = 0; q < B_DMA; ++q) dma16(bk, ob[q], sb + q * 4096);
    };

    // Fragments: lane l supplies row (l % 32) of a 32-row tile and, for sub-step s, the 32
    // bytes k = 64*s + 32*(l/32) .. +31 of the slab, i.e. chunks 4s + 2*(l/32) and the next.
    // A fragment is fetched as two 16-byte LDS reads ("halves").  Fragment f of a sub-step is
    // A tile f for f < MT and B tile f - MT otherwise.
    const int frow = lane & 31, fkb = lane >> 5;
    const int fsw = (frow >> 1) & 7;
    const int a_base = (wm * WTM + frow) * BK;
    const int b_base = A_BYTES + (wn * WTN + frow) * BK;
    constexpr int F = MT + NT;   // fragments per sub-step
    constexpr int NM = MT * NT;  // MFMAs per sub-step
    struct Frags {
        i32x4 h[F][2];
    };
    auto read_half = [&](int kstage, int sub, int f, int half, Frags &fr) {
        const uint8_t *s = lds + (kstage % NSTAGE) * STAGE;
        if ((f < MT && ATN) || (f >= MT && BTN)) {
            // Transposing LDS reads: the 16 lanes of a group each name 8 bytes ("row" t of a
            // 16x8 block), and lane l of the group receives, as byte b, byte l%8 of row
            // 2b + l/8.  With row t = contraction index k0 + t/2, tile rows m0 + 8*(t%2) .. +7,
            // lane l ends up with contraction indices k0 .. k0+7 of tile row m0 + l.  Four such
            // reads make the 32 bytes a lane feeds to one MFMA.
            const int t = lane & 15;
            const int m = (f < MT ? wm * WTM + f * 32 : wn * WTN + (f - MT) * 32) + (frow & 16);
            const bool narrow = f < MT ? BM == 64 : BN == 64;  // one panel of 64-byte rows
            const int obase = (f < MT ? 0 : A_BYTES) + (narrow ? 0 : (m >> 7) * 16384);
            const int mc = narrow ? (m & 63) >> 4 : (m & 127) >> 4;
            i32x2 part[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int k = 64 * sub + 32 * fkb + 8 * (2 * half + e) + (t >> 1);
                const int off = obase + (narrow ? k * 64 + ((mc ^ (((k >> 2) & 1) << 1)) << 4)
                                                : k * 128 + ((mc ^ (((k >> 1) & 3) << 1)) << 4)) + 8 * (t & 1);
                part[e] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                    (__attribute__((address_space(3))) i32x2 *)(s + off));
            }
            fr.h[f][half] = i32x4{part[0].x, part[0].y, part[1].x, part[1].y};
        } else {
            const int chunk = ((4 * sub + 2 * fkb + half) ^ fsw) * 16;
            const int base = f < MT ? a_base + f * 32 * BK : b_base + (f - MT) * 32 * BK;
            fr.h[f][half] = *reinterpret_cast<const i32x4 *>(s + base + chunk);
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // MFMA m of a sub-step works on tile (m / NT, m % NT).
    auto mfma = [&](const Frags &fr, int m) {
        const int i = m / NT, j = m % NT;
        const i32x8 av = __builtin_shufflevector(fr.h[i][0], fr.h[i][1], 0, 1, 2, 3, 4, 5, 6, 7);
        const i32x8 bv =
            __builtin_shufflevector(fr.h[MT + j][0], fr.h[MT + j][1], 0, 1, 2, 3, 4, 5, 6, 7);
        // cbsz = blgp = 1 selects the (1,5,2) format for both operands; the scale operands are
        // zero, i.e. the unscaled instruction.  b goes in as the "row" matrix so that a lane
        // ends up with consecutive output columns.
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv, av, acc[i][j], 1, 1, 0, 0, 0, 0);
    };
    auto issue_one = [&](int kstage, int q) {  // load q (0 .. G-1) of a stage
        const uint32_t sa = lds0 + (kstage % NSTAGE) * STAGE + wave * 1024;
        if (q < A_DMA)
            dma16(a_stage(kstage), oa[q < A_DMA ? q : 0], sa + q * 4096);
        else
            dma16(b_stage(kstage), ob[q >= A_DMA ? q - A_DMA : 0],
                  sa + A_BYTES + (q - A_DMA) * 4096);
    };

    // Wait for this wave's loads of stage t+1 (and for its own LDS reads).  Loads complete in
    // issue order; the groups still allowed in flight are the later stages already issued.
    auto wait_stage = [&](int t) {
        int later = ks_count - 2 - t;  // stages after t+1 that exist
        later = later < NSTAGE - 2 ? later : NSTAGE - 2;
        if (NSTAGE > 2 && later >= NSTAGE - 2) wait_vm_lds<G * (NSTAGE - 2)>();
        else if (NSTAGE > 3 && later == NSTAGE - 3) wait_vm_lds<G * (NSTAGE > 3 ? NSTAGE - 3 : 0)>();
        else wait_vm_lds<0>();
    };

    // The order in which the fragments of a sub-step are fetched: the order in which the
    // MFMAs first need them (B0, A0, B1, ..., then the remaining A tiles).
    auto frag_order = [&](int n) -> int {  // n-th fragment to fetch
        if (n == 0) return MT;             // B0
        if (n == 1) return 0;              // A0
        if (n < NT + 1) return MT + n - 1; // B1 .. B(NT-1)
        return n - NT;                     // A1 .. A(MT-1)
    };

    Frags f0, f1;
    MP8_STAMP_PHASE(1);
    // prologue: fill the ring, fetch the fragments of (0, 0)
#pragma unroll
    for (int st = 0; st < NSTAGE; ++st)
        if (st < ks_count) issue_loads(st);
    wait_stage(-1);
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 2 * F; ++n) read_half(0, 0, frag_order(n / 2), n & 1, f0);
    MP8_STAMP_PHASE(2);
    MP8_BLOCK_STAMP(1);

    // One stage = 2*NM "slots", one MFMA each, fenced so that the order below is the issue
    // order.  Everything else a stage needs is spread over the slots so that it issues in the
    // shadow of the running MFMA (one LDS read costs about a third, one direct load about
    // two thirds of an MFMA's 64 cycles of issue time):
    //   slots 0 .. NM/2-3      the 2F half-fragment reads of sub-step 1 (set f1), early enough
    //                          to have returned when the barrier is reached
    //   end of slot NM/2-1     wait + barrier: stage t+1 has landed everywhere, and nobody
    //                          reads the buffer of stage t any more
    //   slots NM/2 ...         the G direct loads of stage t+NSTAGE, one per slot
    //   slots NM .. 2NM-1      the 2F half-fragment reads of (t+1, sub-step 0) (set f0),
    //                          one per slot from the first slot after set f0's last use
    constexpr int S_BAR = NM / 2 > 0 ? NM / 2 : 1;            // slots before the barrier
    constexpr int S_RD = S_BAR > 2 ? S_BAR - 2 : 1;           // early slots that carry reads
    constexpr int R0 = (2 * F + S_RD - 1) / S_RD;             // half reads per early slot
    constexpr int R1 = (2 * F + NM - 1) / NM;                 // half reads per late slot
    constexpr int D1 = (G + (2 * NM - S_BAR) - 1) / (2 * NM - S_BAR);  // loads per slot
    // Mid-sized tiles with a three-stage ring split the barrier in two (measured +7-11 % there,
    // nothing on the 256x256 tile): the first (end of slot S_BAR-1) only says that nobody reads
    // the buffer of stage t any more, so the loads of stage t+NSTAGE can start; the wait for
    // stage t+1 to land moves to the end of slot NM-1, right before its first fragment read,
    // which gives the loads half a stage more to arrive.  By then N_ISS loads of stage
    // t+NSTAGE are already in flight behind the ones waited for.
    constexpr bool SPLIT_BAR = NM >= 8 && NSTAGE == 3;
    constexpr int N_ISS = (NM - S_BAR) * D1 < G ? (NM - S_BAR) * D1 : G;
    static_assert(!SPLIT_BAR || G * (NSTAGE - 2) + N_ISS < 64, "vmcnt range");
    auto wait_stage_late = [&](int t, bool more_) {
        const int later = ks_count - 2 - t;  // stages after t+1 that exist
        if (more_) wait_vm_lds<SPLIT_BAR ? G * (NSTAGE - 2) + N_ISS : 0>();
        else if (NSTAGE > 2 && later >= NSTAGE - 2) wait_vm_lds<G * (NSTAGE - 2)>();
        else wait_vm_lds<0>();
    };
    for (int t = 0; t < ks_count; ++t) {
        MP8_STAMP(0);
        const bool more = t + NSTAGE < ks_count;
        const bool next = t + 1 < ks_count;
#pragma unroll
        for (int k = 0; k < 2 * NM; ++k) {
            if (k < NM) mfma(f0, k); else mfma(f1, k - NM);
            if (k < S_RD) {
#pragma unroll
                for (int r = 0; r < R0; ++r) {
                    const int n = k * R0 + r;
                    if (n < 2 * F) read_half(t, 1, frag_order(n / 2), n & 1, f1);
                }
            }
            if (k == S_BAR - 1) {
                __builtin_amdgcn_sched_barrier(0);
                MP8_STAMP(1);
                if constexpr (SPLIT_BAR) wait_vm_lds<63>();  // own LDS reads only
                else wait_stage(t);
                MP8_STAMP(2);
                __syncthreads();
                MP8_STAMP(3);
            }
            if (k >= S_BAR) {
#pragma unroll
                for (int r = 0; r < D1; ++r) {
                    const int q = (k - S_BAR) * D1 + r;
                    if (q < G && more) issue_one(t + NSTAGE, q);
                }
            }
            if (k >= NM) {
#pragma unroll
                for (int r = 0; r < R1; ++r) {
                    const int n = (k - NM) * R1 + r;
                    if (n < 2 * F && next) read_half(t + 1, 0, frag_order(n / 2), n & 1, f0);
                }
            }
            if (SPLIT_BAR && k == NM - 1) {  // after this slot's loads: N_ISS are in flight
                __builtin_amdgcn_sched_barrier(0);
                wait_stage_late(t, more);
                __syncthreads();
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        MP8_STAMP(5);
    }
    wait_vm_lds<0>();
    MP8_STAMP_PHASE(3);
    MP8_BLOCK_STAMP(2);

    // Epilogue.  acc[i][j][4g + e] is output row  wm*WTM + 32i + lane%32  and column
    // wn*WTN + 32j + 8g + 4*(lane/32) + e.  Each wave passes its tile through LDS one band
    // of 32 rows at a time, so that afterwards every lane owns 16 consecutive columns of one
    // row: full 16-byte stores of codes, 64-byte runs of FP32, one Philox block per eight
    // elements.
    constexpr int EP_LD = WTN + 4;                 // floats per band row (+4: bank spread)
    constexpr int CG = WTN / 16;                   // 16-column groups per band row
    constexpr int BANDS = MT >= 2 ? 2 : 1;         // bands staged per pass
    static_assert(4 * BANDS * 32 * EP_LD * 4 <= LDS_BYTES, "band buffers fit in LDS");
    __syncthreads();                               // all waves are done with the operand ring
    if constexpr (EPI == EPI_RNE) {
        // RNE only: convert in registers (four codes = one register), join the two half-wave
        // column sets of every 32x32 tile with two v_permlane32_swap -- lane (row, h) then
        // holds the 16-byte piece of columns 32j + 16h .. +15 -- and collect the whole block
        // tile of codes (BM x BN bytes) in LDS, piece q of row r in slot q ^ f(r) with
        // f(r) = (r / rows per 256 bytes) mod pieces per row: conflict-free for the writes
        // (16 rows, one piece) and for the reads (consecutive pieces of a row).  Then the
        // block stores whole rows of the tile: BN / 16 consecutive lanes per row.
        constexpr int NP = BN / 16;                // pieces per tile row
        constexpr int RP = 256 / BN > 0 ? 256 / BN : 1;  // tile rows per 256 bytes of LDS
        static_assert(BM * BN <= LDS_BYTES, "code tile fits in LDS");
        auto slot = [&](int r, int q) { return r * BN + ((q ^ ((r / RP) & (NP - 1))) << 4); };
        auto tiles = [&](auto unit_alpha) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    uint32_t pk[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float y[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                      acc[i][j][4 * g + 3]};
                        if constexpr (!decltype(unit_alpha)::value) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) y[e] *= p.ep.alpha;
                        }
                        pk[g] = e5m2_pack4<false>(y, 0u, 0u, false);
                    }
                    // after swap(pk[g], pk[g+2]): lower half = own columns 8g .. 8g+3 and the
                    // upper half's 8g+4 .. 8g+7; upper half = the lower half's 16+8g .. +3 and
                    // its own 16+8g+4 .. +7
                    const auto s0 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
                    u32x4 o = {s0[0], s0[1], s1[0], s1[1]};
                    *reinterpret_cast<u32x4 *>(lds + slot(wm * WTM + 32 * i + frow,
                                                          (wn * WTN + 32 * j) / 16 + fkb)) = o;
                }
        };
        if (p.ep.alpha == 1.0f) tiles(std::true_type{});
        else tiles(std::false_type{});
        __syncthreads();
        const int q = threadIdx.x % NP;
        const int64_t c = col0 + 16 * q;
#pragma unroll
        for (int k = 0; k < BM * NP / 256; ++k) {
            const int rr = k * (256 / NP) + threadIdx.x / NP;
            u32x4 o = *reinterpret_cast<const u32x4 *>(lds + slot(rr, q));
            const int64_t r = row0 + rr;
            if (r < p.rows && c < p.cols) {
                if (p.ep.mask && conv_padding_row(p.ep, r)) o = u32x4{0u, 0u, 0u, 0u};
                *reinterpret_cast<u32x4 *>(p.ep.out8 + r * p.cols + c) = o;
            }
        }
        MP8_STAMP_PHASE(4);
        MP8_BLOCK_STAMP(3);
        return;
    }
    float *band = reinterpret_cast<float *>(lds) + wave * BANDS * 32 * EP_LD;
    StatsAcc st;
    const bool fast_cols = (p.cols & 15) == 0;
#pragma unroll
    for (int h = 0; h < MT; h += BANDS) {
#pragma unroll
        for (int bi = 0; bi < BANDS; ++bi)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 o = {acc[h + bi][j][4 * g], acc[h + bi][j][4 * g + 1],
                               acc[h + bi][j][4 * g + 2], acc[h + bi][j][4 * g + 3]};
                    *reinterpret_cast<f32x4 *>(band + (32 * bi + frow) * EP_LD + 32 * j + 8 * g +
                                               4 * fkb) = o;
                }
        // the bands are private to this wave: order the LDS writes before the reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        MP8_STAMP_PHASE(5);
        // the RNE-only variant is small enough to unroll: the LDS reads of several items then
        // overlap instead of each item paying the full LDS latency
#pragma unroll(EPI == EPI_RNE ? 4 : 1)
        for (int item = lane; item < BANDS * 32 * CG; item += 64) {
            const int br = item / CG, cg = item - br * CG;
            const int64_t r = row0 + wm * WTM + 32 * h + br;
            const int64_t c = col0 + wn * WTN + 16 * cg;
            if (r < p.rows && c < p.cols) {
                float v[16];
                const f32x4 *src = reinterpret_cast<const f32x4 *>(band + br * EP_LD + 16 * cg);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 x = src[q];
                    v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
                }
                emit16<EPI>(p, split, r, c, v, st, fast_cols);
            }
        }
        MP8_STAMP_PHASE(6);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
    MP8_STAMP_PHASE(4);
    MP8_BLOCK_STAMP(3);
}

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
// row), else 0.
template <int EPI, bool ATN, bool BTN, int CONV>
__global__ __launch_bounds__(256, 1) void gemm_wavek_kernel(const GemmArgs p) {
    static_assert(CONV == 0 || (CONV == 3 && ATN && BTN), "plain or convolution weight gradient");
    static_assert(BTN || !ATN, "a alone contraction-major is not built");
    constexpr int BM = 64, BN = 64;
    constexpr int SLAB = 64 * BK;           // 64 rows of 128 bytes, or 128 contraction rows of 64
    constexpr int STAGE = 2 * SLAB;         // a, then b
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
    auto issue = [&](int j) {  // stage j of this wave into buffer j % 2: 16 loads
        const uint8_t *ak = a_tile + (int64_t)(4 * j) * a_kstep;
        const uint8_t *bk = b_tile + (int64_t)(4 * j) * b_kstep;
        const uint32_t sa = ring0 + (j & 1) * STAGE;
#pragma unroll
        for (int q = 0; q < 8; ++q) dma16(ak, oa[q], sa + q * 1024);
#pragma unroll
        for (int q = 0; q < 8; ++q) dma16(bk, ob[q], sa + SLAB + q * 1024);
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    const int frow = lane & 31, fkb = lane >> 5, t16 = lane & 15;
    // fragment f (0, 1: a tile rows 32f ..; 2, 3: b) of half stage `sub` from buffer `s`: lane l
    // supplies tile row 32f + l%32 and contraction indices 64*sub + 32*(l/32) .. +31 -- two
    // 16-byte reads of a row-major slab, four transposing reads of eight contraction indices
    // each of a contraction-major one (see the general kernel)
    auto fragment = [&](const uint8_t *s, int sub, int f) -> i32x8 {
        const uint8_t *slab = s + (f >> 1) * SLAB;
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
        if (j + 1 < mine) wait_vm_lds<16>();  // the sixteen loads of the next stage may fly
        else wait_vm_lds<0>();
        const uint8_t *s = ring + (j & 1) * STAGE;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const i32x8 a0 = fragment(s, sub, 0), a1 = fragment(s, sub, 1);
            const i32x8 b0 = fragment(s, sub, 2), b1 = fragment(s, sub, 3);
            // bf8 x bf8, unscaled; b as the "row" matrix: a lane gets consecutive output columns
            acc[0][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b0, a0, acc[0][0], 1, 1, 0, 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b1, a0, acc[0][1], 1, 1, 0, 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b0, a1, acc[1][0], 1, 1, 0, 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b1, a1, acc[1][1], 1, 1, 0, 0, 0, 0);
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
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                *reinterpret_cast<f32x4 *>(red + (wave * BM + 32 * i + frow) * RED_LD + 32 * j + 8 * g + 4 * fkb) = o;
            }
    __syncthreads();
    StatsAcc st;
    const bool fast_cols = (p.cols & 15) == 0;
    {
        const int rr = threadIdx.x >> 2, cg = threadIdx.x & 3;
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
    MP8_BLOCK_STAMP(0);
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
            if (st == 0) MP8_BLOCK_STAMP(1);
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
    MP8_BLOCK_STAMP(2);
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
        MP8_BLOCK_STAMP(3);
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

// Finish four consecutive columns c .. c+3 (c % 4 == 0, row length a multiple of 4).
__device__ __forceinline__ uint32_t finish4(const Epilogue &ep, int64_t r, int64_t c, float v[4],
                                            StatsAcc &st) {
    const int64_t i0 = r * ep.cols + c;
    if (ep.acc_mode != 0) {
        f32x4 *p = reinterpret_cast<f32x4 *>(ep.acc + i0);
        if (ep.acc_mode == 2) {
            f32x4 o = *p;
            v[0] += o.x; v[1] += o.y; v[2] += o.z; v[3] += o.w;
        }
        f32x4 n = {v[0], v[1], v[2], v[3]};
        *p = n;
    }
    if (ep.out8 == nullptr && ep.out8_t == nullptr && ep.stats == nullptr && !ep.want_codes) return 0;
    uint32_t r01 = 0, r23 = 0;
    if (ep.sr) {
        // elements i0..i0+3 are halfwords (i0 % 8) .. +3 of Philox block i0 / 8
        const Philox rng(ep.seed, ep.offset);
        uint4 w = rng.block((uint64_t)i0 >> 3);
        r01 = (i0 & 4) ? w.z : w.x;
        r23 = (i0 & 4) ? w.w : w.y;
    }
    float y[4] = {v[0] * ep.alpha, v[1] * ep.alpha, v[2] * ep.alpha, v[3] * ep.alpha};
    uint32_t pk = e5m2_pack4_rt(y, r01, r23, ep.sr != 0, ep.sat != 0);
    if (ep.mask && conv_padding_row(ep, r)) pk = 0;
    else if (ep.stats != nullptr) st.add4(y, pk);
    if (ep.out8 != nullptr) *reinterpret_cast<uint32_t *>(ep.out8 + i0) = pk;
    if (ep.out8_t != nullptr) {
        uint8_t *t = ep.out8_t + c * ep.rows + r;
        t[0] = (uint8_t)pk;
        t[ep.rows] = (uint8_t)(pk >> 8);
        t[2 * ep.rows] = (uint8_t)(pk >> 16);
        t[3 * ep.rows] = (uint8_t)(pk >> 24);
    }
    return pk;
}

// Optional second half of Figure 1b in the finishing pass: the 8-bit weight gradient that was
// just rounded is un-scaled and applied to the half-precision master weights, exactly as
// mp8_sgd_update_fp16_sr would do it from memory (same arithmetic, same random stream: element
// i uses halfword i % 8 of block i / 8 of the update's own Philox stream).  w16 == nullptr:
// no update.
struct UpdateHook {
    uint16_t *w16;
    uint8_t *w8_out;
    const uint32_t *skip;
    float neg_lr, inv_scale;
    int sr;
    uint64_t seed, offset;
};

__device__ __forceinline__ void update_element(const UpdateHook &u, int64_t i, uint32_t code, uint32_t r16) {
    const uint32_t h = u.sr ? update_one<true>(u.w16[i], code, u.neg_lr, u.inv_scale, r16)
                            : update_one<false>(u.w16[i], code, u.neg_lr, u.inv_scale, 0u);
    u.w16[i] = (uint16_t)h;
    if (u.w8_out != nullptr) u.w8_out[i] = (uint8_t)e5m2_of_half(h);
}

// Elements i0 .. i0+3 (i0 % 4 == 0) from their four packed gradient codes.
__device__ __forceinline__ void update4(const UpdateHook &u, int64_t i0, uint32_t pk) {
    uint32_t r01 = 0, r23 = 0;
    if (u.sr) {
        const Philox rng(u.seed, u.offset);
        const uint4 w = rng.block((uint64_t)i0 >> 3);
        r01 = (i0 & 4) ? w.z : w.x;
        r23 = (i0 & 4) ? w.w : w.y;
    }
    u32x2 *wp = reinterpret_cast<u32x2 *>(u.w16 + i0);
    const u32x2 wr = *wp;
    uint32_t h[4];
    const uint32_t w16v[4] = {wr.x & 0xFFFFu, wr.x >> 16, wr.y & 0xFFFFu, wr.y >> 16};
    const uint32_t r16[4] = {r01 & 0xFFFFu, r01 >> 16, r23 & 0xFFFFu, r23 >> 16};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t code = (pk >> (8 * j)) & 0xFFu;
        h[j] = u.sr ? update_one<true>(w16v[j], code, u.neg_lr, u.inv_scale, r16[j])
                    : update_one<false>(w16v[j], code, u.neg_lr, u.inv_scale, 0u);
    }
    const u32x2 o = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
    *wp = o;
    if (u.w8_out != nullptr)
        *reinterpret_cast<uint32_t *>(u.w8_out + i0) =
            e5m2_of_half(h[0]) | (e5m2_of_half(h[1]) << 8) | (e5m2_of_half(h[2]) << 16) | (e5m2_of_half(h[3]) << 24);
}

// Sum the FP32 tiles of the contraction slices in slice order and finish: the complete sum is
// rounded once.  One thread per four columns (per element when the row length is not a
// multiple of four).
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float *__restrict__ partial,
                                                            int splits, const Epilogue ep,
                                                            const UpdateHook upd) {
    StatsAcc st;
    // an overflowed step leaves the master weights alone (the gradient codes are still written)
    const bool updating = upd.w16 != nullptr && !(upd.skip != nullptr && *upd.skip != 0u);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t slice = ep.rows * ep.cols;
    if ((ep.cols & 3) == 0) {
        const int64_t total = slice >> 2;
        for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += stride) {
            const int64_t i0 = t << 2;
            const int64_t r = i0 / ep.cols, c = i0 - r * ep.cols;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            int s = 0;
            for (; s + 4 <= splits; s += 4) {  // four loads in flight, added in slice order
                f32x4 x0 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)s * slice + i0);
                f32x4 x1 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(s + 1) * slice + i0);
                f32x4 x2 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(s + 2) * slice + i0);
                f32x4 x3 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(s + 3) * slice + i0);
                v[0] += x0.x; v[1] += x0.y; v[2] += x0.z; v[3] += x0.w;
                v[0] += x1.x; v[1] += x1.y; v[2] += x1.z; v[3] += x1.w;
                v[0] += x2.x; v[1] += x2.y; v[2] += x2.z; v[3] += x2.w;
                v[0] += x3.x; v[1] += x3.y; v[2] += x3.z; v[3] += x3.w;
            }
            for (; s < splits; ++s) {
                f32x4 x = *reinterpret_cast<const f32x4 *>(partial + (int64_t)s * slice + i0);
                v[0] += x.x; v[1] += x.y; v[2] += x.z; v[3] += x.w;
            }
            const uint32_t pk = finish4(ep, r, c, v, st);
            if (updating) update4(upd, i0, pk);
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < slice; i += stride) {
            float v = 0.f;
            for (int s = 0; s < splits; ++s) v += partial[(int64_t)s * slice + i];
            const int64_t r = i / ep.cols;
            const uint32_t code = finish1(ep, r, i - r * ep.cols, v, st);
            if (updating) {
                uint32_t r16 = 0;
                if (upd.sr) {
                    const Philox rng(upd.seed, upd.offset);
                    r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
                }
                update_element(upd, i, code, r16);
            }
        }
    }
    if (ep.stats != nullptr) st.flush(ep.stats);
}

// Any-shape fallback: one thread per output element, operands decoded one by one, FP32 fused
// multiply-adds in contraction order.  Used when the contraction length is not a multiple of
// 128 or the operands are not 16-byte aligned.
__global__ __launch_bounds__(256) void gemm_generic_kernel(const uint8_t *__restrict__ a,
                                                           int64_t lda,
                                                           const uint8_t *__restrict__ b,
                                                           int64_t ldb, int64_t kc, int tn,
                                                           const Epilogue ep) {
    const int64_t total = ep.rows * ep.cols;
    StatsAcc st;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t r = t / ep.cols, c = t - r * ep.cols;
        // element (r, j) of a: a[r * lda + j], or a[j * lda + r] when a is contraction-major
        // (bit 0 of tn; bit 1 likewise for b)
        const uint8_t *ar = (tn & 1) ? a + r : a + r * lda, *bc = (tn & 2) ? b + c : b + c * ldb;
        const int64_t sa = (tn & 1) ? lda : 1, sb = (tn & 2) ? ldb : 1;
        float s = 0.f;
        for (int64_t j = 0; j < kc; ++j)
            s = __builtin_fmaf(e5m2_to_f32(ar[j * sa]), e5m2_to_f32(bc[j * sb]), s);
        finish1(ep, r, c, s, st);
    }
    if (ep.stats != nullptr) st.flush(ep.stats);
}

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
static const TileConfig kTiles[] = {
    MP8_TILE_TN(256, 256, 2, 2, 2, 1), MP8_TILE(256, 128, 2, 2, 3, 1), MP8_TILE(128, 256, 2, 2, 3, 1),
    MP8_TILE_TN(128, 128, 2, 2, 2, 2), MP8_TILE_TN(128, 128, 2, 2, 4, 1), MP8_TILE(64, 128, 1, 4, 3, 2),
    MP8_TILE(128, 64, 4, 1, 3, 2),  MP8_TILE_TN(64, 64, 2, 2, 4, 2), MP8_TILE(64, 128, 1, 4, 2, 3),
    MP8_TILE(128, 64, 4, 1, 2, 3),  MP8_TILE_TN(64, 64, 2, 2, 2, 4),   MP8_TILE_SHORTK,
    MP8_TILE_WAVEK,
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
enum { T256x256 = 0, T128x128s2 = 3, T128x128s4 = 4, T128x64s2 = 9, T64x64s2 = 10, T128x128k = 11, T64x64w = 12 };
static Plan make_plan(int64_t rows, int64_t cols, int64_t kc, int tile_config, int split_k,
                      int layout = 0) {  // bit 0: a contraction-major, bit 1: b
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
        if (n256 >= 208 && fill256 >= 0.8 && ksteps >= 8) t = T256x256;
        else if (n64 <= kCUs && ksteps >= 16) t = T64x64w;  // one workgroup per CU, one round
        else if (tn && (n128 < 16 || (n128 < 192 && ksteps <= 64))) t = T64x64s2;
        else if (tn) t = ksteps >= 64 ? T128x128s4 : T128x128s2;
        else if (n128 >= 192 && ksteps <= 2) t = T128x128k;  // all prologue and epilogue
        else if (n128 >= 192) t = (ksteps >= 64 && n128 <= 2 * kCUs) ? T128x128s4 : T128x128s2;
        else t = T64x64s2;
    }
    pl.tile = t;
    pl.tiles_m = (int)((rows + kTiles[t].bm - 1) / kTiles[t].bm);
    pl.tiles_n = (int)((cols + kTiles[t].bn - 1) / kTiles[t].bn);
    const int64_t nt = (int64_t)pl.tiles_m * pl.tiles_n;
    int s = 1;
    if (kTiles[t].max_ksteps > 0) {
        s = 1;  // these kernels take the whole contraction at once
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
                              size_t workspace_bytes, hipStream_t s, const UpdateHook *upd = nullptr) {
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
            hipLaunchKernelGGL(splitk_finish_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                               (const float *)partial, pl.splits, fin, upd ? *upd : UpdateHook{});
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
                            void *stream, int tile_config, int split_k, const UpdateHook *upd) {
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
                       workspace_bytes, s, upd);
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
    UpdateHook upd{};
    upd.w16 = w16;
    upd.w8_out = w8_out;
    upd.skip = skip_if_nonzero;
    upd.neg_lr = -lr;
    upd.inv_scale = inv_loss_scale;
    upd.sr = w_round == MP8_SR;
    upd.seed = w_seed;
    upd.offset = w_offset;
    const mp8_status st = gemm_impl(MP8_WGRAD, M, N, K, a, lda, b, ldb, alpha, nullptr, 0, g8_out, nullptr,
                                    g_round, flags, g_seed, g_offset, stats, workspace, workspace_bytes,
                                    stream, 0, 0, &upd);
    if (st != MP8_ERR_UNSUPPORTED || g8_out == nullptr) return st;
    // shapes that only the any-shape kernel takes: two launches through the 8-bit gradient
    const mp8_status sg = mp8_gemm_fp8(MP8_WGRAD, M, N, K, a, lda, b, ldb, alpha, nullptr, 0, g8_out, nullptr,
                                       g_round, flags, g_seed, g_offset, stats, workspace, workspace_bytes,
                                       stream);
    if (sg != MP8_OK) return sg;
    return mp8_sgd_update_fp16_sr(w16, g8_out, K * N, lr, inv_loss_scale, w_round, w_seed, w_offset,
                                  skip_if_nonzero, w8_out, nullptr, stream);
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

static Plan conv_plan(mp8_op op, const ConvDims &d, int64_t Ci) {
    // the tile shapes built for contraction-major operands are the ones built for convolutions
    Plan pl = make_plan(d.rows, d.cols, d.kc, 0, 0, 3);
    // a tile row of the weight gradient must not straddle two taps
    if (pl.mfma && op == MP8_WGRAD && (Ci % kTiles[pl.tile].bm) != 0)
        pl = make_plan(d.rows, d.cols, d.kc, T128x128s2 + 1, 0, 3);
    // forward and backward data have one tile row per 128 pixels and few tile columns: the
    // 128-row tile keeps the re-reads of the weights low
    if (pl.mfma && op != MP8_WGRAD && kTiles[pl.tile].bm < 128)
        pl = make_plan(d.rows, d.cols, d.kc, T128x128s2 + 1, 0, 3);
    return pl;
}

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
    // whole 128-byte stages per tap, whole tiles per tap of the weight gradient
    if ((Ci & 127) != 0 || (Co & 127) != 0 || Ci >= (1 << 20) || Co >= (1 << 20)) return MP8_ERR_UNSUPPORTED;
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
    ga.cv.div_cpb = make_fastdiv((uint32_t)((op == MP8_BWD_DATA ? Co : Ci) / 128));
    ga.cv.b_tap_stride = Ci * Co;
    ga.cv.div_ci = make_fastdiv((uint32_t)Ci);
    return launch_mfma(ga, ep, pl, d.kc, kTiles[pl.tile].kernel_conv[(int)op], workspace, workspace_bytes,
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
    UpdateHook upd{};
    upd.w16 = w16;
    upd.w8_out = w8_out;
    upd.skip = skip_if_nonzero;
    upd.neg_lr = -lr;
    upd.inv_scale = inv_loss_scale;
    upd.sr = w_round == MP8_SR;
    upd.seed = w_seed;
    upd.offset = w_offset;
    return conv_impl(MP8_WGRAD, B, H, W, Ci, Co, prows, x8, e8, alpha, nullptr, 0, g8_out, g_round, flags,
                     g_seed, g_offset, stats, workspace, workspace_bytes, stream, &upd);
}

#ifdef MP8_TRACE
extern "C" int mp8_debug_read_trace(unsigned long long *host, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(mp8::mp8_trace_buf), bytes);
}
extern "C" int mp8_debug_read_block_times(unsigned long long *host, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(mp8::mp8_block_times), bytes);
}
#endif
