// mp8_quantize_e5m2 / mp8_sr_bits: the Q node of Figure 1a (arXiv 1905.12334, Section 3)
// as HBM-streaming kernels for gfx950.
//
// Flat kernel: every lane owns groups of 16 consecutive elements (64 B of FP32 in, 16 B of
// codes out), which is also two groups of eight for the random-bit stream (one Philox block
// per eight elements).  Transposing kernel: a 64x64 tile goes through LDS so that both the
// row-major and the transposed copy are written with full 16-byte stores.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "mp8_device.hpp"

namespace mp8 {

template <bool kF16>
__device__ __forceinline__ float load_src(const void *src, int64_t i) {
    if constexpr (kF16)
        return __half2float(reinterpret_cast<const __half *>(src)[i]);
    else
        return reinterpret_cast<const float *>(src)[i];
}

// Load eight consecutive source elements starting at i (i % 8 == 0, all in range).
template <bool kF16>
__device__ __forceinline__ void load8(const void *src, int64_t i, float v[8]) {
    if constexpr (kF16) {
        uint4 raw = *reinterpret_cast<const uint4 *>(reinterpret_cast<const __half *>(src) + i);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float2 f = __half22float2(h[j]);
            v[2 * j] = f.x;
            v[2 * j + 1] = f.y;
        }
    } else {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(src) + i);
        f32x4 x0 = __builtin_nontemporal_load(p);
        f32x4 x1 = __builtin_nontemporal_load(p + 1);
        v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
        v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
    }
}

// Round eight scaled values that share Philox block `blk`; returns the codes packed
// little-endian (element 0 in the low byte of .x).
template <bool kSR, bool kStats>
__device__ __forceinline__ uint2 round8(const float v[8], float scale, bool sat,
                                        const Philox &rng, uint64_t blk, StatsAcc &st) {
    uint4 w = make_uint4(0, 0, 0, 0);
    if constexpr (kSR) w = rng.block(blk);
    const uint32_t rw[4] = {w.x, w.y, w.z, w.w};
    uint32_t c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t u = f2u(v[j] * scale);
        uint32_t r16 = (j & 1) ? (rw[j >> 1] >> 16) : (rw[j >> 1] & 0xFFFFu);
        c[j] = e5m2_from_f32_bits<kSR>(u, r16, sat);
        if constexpr (kStats) st.add(u & 0x7FFFFFFFu, c[j]);
    }
    uint2 o;
    o.x = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
    o.y = c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24);
    return o;
}

template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(256) void quantize_flat_kernel(const void *__restrict__ src,
                                                            uint8_t *__restrict__ dst, int64_t n,
                                                            float scale, int sat, uint64_t seed,
                                                            uint64_t offset, mp8_stats *stats) {
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t ngroups = n >> 4;  // full groups of 16 elements
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < ngroups; g += stride) {
        float v[16];
        load8<kF16>(src, g * 16, v);
        load8<kF16>(src, g * 16 + 8, v + 8);
        uint2 lo = round8<kSR, kStats>(v, scale, sat != 0, rng, (uint64_t)(2 * g), st);
        uint2 hi = round8<kSR, kStats>(v + 8, scale, sat != 0, rng, (uint64_t)(2 * g + 1), st);
        u32x4 pk = {lo.x, lo.y, hi.x, hi.y};
        __builtin_nontemporal_store(pk, reinterpret_cast<u32x4 *>(dst + g * 16));
    }
    // ragged tail (< 16 elements): one element per lane of the first wave of block 0
    if (blockIdx.x == 0 && threadIdx.x < 16) {
        int64_t i = (ngroups << 4) + threadIdx.x;
        if (i < n) {
            uint32_t u = f2u(load_src<kF16>(src, i) * scale);
            uint32_t r16 = 0;
            if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
            uint32_t c = e5m2_from_f32_bits<kSR>(u, r16, sat != 0);
            dst[i] = (uint8_t)c;
            if constexpr (kStats) st.add(u & 0x7FFFFFFFu, c);
        }
    }
    if constexpr (kStats) st.flush(stats);
}

// 64x64 tile per block of 256 threads.  Thread t handles row (t / 4) + {0}, 16 columns
// starting at 16 * (t % 4): codes are packed into a uint4, written to dst directly and into
// an LDS tile; after the barrier the tile is read column-wise for the transposed copy.
template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(256) void quantize_transpose_kernel(
    const void *__restrict__ src, uint8_t *__restrict__ dst, uint8_t *__restrict__ dst_t,
    int64_t rows, int64_t cols, float scale, int sat, uint64_t seed, uint64_t offset,
    mp8_stats *stats) {
    constexpr int T = 64;
    // rows of 17 dwords: the column reads of the transposed pass spread over the banks
    __shared__ __attribute__((aligned(16))) uint8_t tile[T][T + 4];
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t tiles_c = (cols + T - 1) / T;
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * T;
    const int64_t c0 = (int64_t)(blockIdx.x % tiles_c) * T;
    const int tr = threadIdx.x >> 2;         // 0..63 row inside the tile
    const int tc = (threadIdx.x & 3) * 16;   // column offset inside the tile
    const int64_t r = r0 + tr, c = c0 + tc;
    const bool fast = ((cols & 15) == 0);    // rows of 16-element groups are aligned
    if (r < rows && c < cols) {
        if (fast) {
            float v[16];
            const int64_t i = r * cols + c;
            load8<kF16>(src, i, v);
            load8<kF16>(src, i + 8, v + 8);
            uint2 lo = round8<kSR, kStats>(v, scale, sat != 0, rng, (uint64_t)i >> 3, st);
            uint2 hi = round8<kSR, kStats>(v + 8, scale, sat != 0, rng, ((uint64_t)i >> 3) + 1, st);
            uint4 pk = make_uint4(lo.x, lo.y, hi.x, hi.y);
            *reinterpret_cast<uint4 *>(dst + i) = pk;
            uint32_t *trow = reinterpret_cast<uint32_t *>(&tile[tr][tc]);
            trow[0] = pk.x; trow[1] = pk.y; trow[2] = pk.z; trow[3] = pk.w;
        } else {
            for (int j = 0; j < 16 && c + j < cols; ++j) {
                const int64_t i = r * cols + c + j;
                uint32_t u = f2u(load_src<kF16>(src, i) * scale);
                uint32_t r16 = 0;
                if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
                uint32_t cd = e5m2_from_f32_bits<kSR>(u, r16, sat != 0);
                if constexpr (kStats) st.add(u & 0x7FFFFFFFu, cd);
                dst[i] = (uint8_t)cd;
                tile[tr][tc + j] = (uint8_t)cd;
            }
        }
    }
    __syncthreads();
    // transposed write: thread t writes 16 consecutive source-rows of source-column tr2
    const int tr2 = threadIdx.x >> 2;        // source column inside the tile
    const int tq = (threadIdx.x & 3) * 16;   // first source row inside the tile
    const int64_t oc = c0 + tr2;             // row of dst_t
    const int64_t orow0 = r0 + tq;           // column of dst_t
    if (oc < cols && orow0 < rows) {
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 16; ++j) w[j >> 2] |= (uint32_t)tile[tq + j][tr2] << (8 * (j & 3));
        uint8_t *p = dst_t + oc * rows + orow0;
        if (((rows & 15) == 0) && orow0 + 16 <= rows) {
            *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            for (int j = 0; j < 16 && orow0 + j < rows; ++j) p[j] = (uint8_t)(w[j >> 2] >> (8 * (j & 3)));
        }
    }
    if constexpr (kStats) st.flush(stats);
}

__global__ __launch_bounds__(256) void sr_bits_kernel(uint16_t *out, int64_t n, uint64_t seed,
                                                      uint64_t offset) {
    const Philox rng(seed, offset);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = (uint16_t)philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
}

template <bool kF16, bool kSR, bool kStats>
static hipError_t launch_quantize(const void *src, uint8_t *dst, uint8_t *dst_t, int64_t rows,
                                  int64_t cols, float scale, int sat, uint64_t seed,
                                  uint64_t offset, mp8_stats *stats, hipStream_t s) {
    const int64_t n = rows * cols;
    if (dst_t == nullptr) {
        int64_t groups = (n >> 4) + 1;
        int64_t blocks = (groups + 255) / 256;
        const int64_t cap = 256 * 16;  // 16 blocks per CU, grid-stride beyond that
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL((quantize_flat_kernel<kF16, kSR, kStats>), dim3((unsigned)blocks),
                           dim3(256), 0, s, src, dst, n, scale, sat, seed, offset, stats);
    } else {
        int64_t tiles = ((rows + 63) / 64) * ((cols + 63) / 64);
        hipLaunchKernelGGL((quantize_transpose_kernel<kF16, kSR, kStats>), dim3((unsigned)tiles),
                           dim3(256), 0, s, src, dst, dst_t, rows, cols, scale, sat, seed, offset,
                           stats);
    }
    return hipGetLastError();
}

}  // namespace mp8

extern "C" mp8_status mp8_quantize_e5m2(const void *src, int src_is_f16, uint8_t *dst,
                                        uint8_t *dst_t, int64_t rows, int64_t cols, float scale,
                                        mp8_round round, int flags, uint64_t seed,
                                        uint64_t offset, mp8_stats *stats, void *stream) {
    using namespace mp8;
    if (rows < 0 || cols < 0) return MP8_ERR_INVALID_ARG;
    if (round != MP8_RNE && round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return MP8_OK;
    if (!src || !dst) return MP8_ERR_INVALID_ARG;
    if (rows > (INT64_MAX / cols)) return MP8_ERR_UNSUPPORTED;
    if (dst_t && ((rows + 63) / 64) * ((cols + 63) / 64) > 0x7FFFFFFFLL) return MP8_ERR_UNSUPPORTED;
    if (((uintptr_t)src | (uintptr_t)dst | (uintptr_t)dst_t) & 15u) return MP8_ERR_ALIGNMENT;
    hipStream_t s = (hipStream_t)stream;
    const int sat = (flags & MP8_FLAG_SATURATE) ? 1 : 0;
    hipError_t e;
#define MP8_Q(F16, SR, ST) \
    e = launch_quantize<F16, SR, ST>(src, dst, dst_t, rows, cols, scale, sat, seed, offset, stats, s)
    const bool f16 = src_is_f16 != 0, sr = round == MP8_SR, st = stats != nullptr;
    if (f16) {
        if (sr) { if (st) MP8_Q(true, true, true); else MP8_Q(true, true, false); }
        else    { if (st) MP8_Q(true, false, true); else MP8_Q(true, false, false); }
    } else {
        if (sr) { if (st) MP8_Q(false, true, true); else MP8_Q(false, true, false); }
        else    { if (st) MP8_Q(false, false, true); else MP8_Q(false, false, false); }
    }
#undef MP8_Q
    return e == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}

extern "C" mp8_status mp8_sr_bits(uint16_t *out, int64_t n, uint64_t seed, uint64_t offset,
                                  void *stream) {
    if (n < 0) return MP8_ERR_INVALID_ARG;
    if (n == 0) return MP8_OK;
    if (!out) return MP8_ERR_INVALID_ARG;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(mp8::sr_bits_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, out, n, seed, offset);
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}
