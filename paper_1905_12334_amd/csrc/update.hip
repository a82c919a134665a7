// mp8_sgd_update_fp16_sr: the weight-update path of Figure 1b (arXiv 1905.12334, Section 3)
// as one HBM-streaming kernel for gfx950.  Per element: the 8-bit gradient is un-scaled in
// FP32, the half-precision master weight is widened to FP32, updated with one fused
// multiply-add and stored back as half with round-to-nearest-even or stochastic rounding.
// 5 bytes of traffic per element (2 + 1 read, 2 written), +1 with the optional 8-bit copy.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "mp8_device.hpp"

namespace mp8 {

template <bool kSR>
__device__ __forceinline__ uint32_t update_one(uint32_t w16, uint32_t g8, float neg_lr,
                                               float inv_scale, uint32_t r16) {
    float g = e5m2_to_f32(g8) * inv_scale;
    float w = __half2float(__ushort_as_half((unsigned short)w16));
    float wn = __builtin_fmaf(neg_lr, g, w);
    return f16_from_f32_bits<kSR>(f2u(wn), r16);
}

// Each lane owns groups of 16 consecutive elements: 32 B of weights in and out, 16 B of
// gradients, two Philox blocks.
template <bool kSR, bool kW8, bool kStats>
__global__ __launch_bounds__(256) void sgd_update_kernel(uint16_t *__restrict__ w16,
                                                         const uint8_t *__restrict__ g8,
                                                         int64_t n, float neg_lr,
                                                         float inv_scale, uint64_t seed,
                                                         uint64_t offset,
                                                         const uint32_t *__restrict__ skip,
                                                         uint8_t *__restrict__ w8_out,
                                                         mp8_stats *stats) {
    const Philox rng(seed, offset);
    const bool skipping = (skip != nullptr) && (*skip != 0u);
    if (skipping && !kStats) return;
    uint32_t nonfinite = 0;
    const int64_t ngroups = n >> 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < ngroups; g += stride) {
        u32x4 gr = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(g8 + g * 16));
        const uint32_t gw[4] = {gr.x, gr.y, gr.z, gr.w};
        if constexpr (kStats) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                nonfinite += ((((gw[j >> 2] >> (8 * (j & 3))) & 0x7Cu) == 0x7Cu) ? 1u : 0u);
        }
        if (skipping) continue;
        u32x4 *wp = reinterpret_cast<u32x4 *>(w16 + g * 16);
        u32x4 wa = wp[0], wb = wp[1];
        uint32_t ww[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
        uint32_t rw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if constexpr (kSR) {
            uint4 r0 = rng.block((uint64_t)(2 * g));
            uint4 r1 = rng.block((uint64_t)(2 * g + 1));
            rw[0] = r0.x; rw[1] = r0.y; rw[2] = r0.z; rw[3] = r0.w;
            rw[4] = r1.x; rw[5] = r1.y; rw[6] = r1.z; rw[7] = r1.w;
        }
        uint32_t w8[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 8; ++j) {  // pair j = elements 2j, 2j+1
            uint32_t g_lo = (gw[j >> 1] >> (16 * (j & 1))) & 0xFFu;
            uint32_t g_hi = (gw[j >> 1] >> (16 * (j & 1) + 8)) & 0xFFu;
            uint32_t h_lo = update_one<kSR>(ww[j] & 0xFFFFu, g_lo, neg_lr, inv_scale, rw[j] & 0xFFFFu);
            uint32_t h_hi = update_one<kSR>(ww[j] >> 16, g_hi, neg_lr, inv_scale, rw[j] >> 16);
            ww[j] = h_lo | (h_hi << 16);
            if constexpr (kW8) {
                uint32_t c_lo = e5m2_from_f32_bits<false>(
                    f2u(__half2float(__ushort_as_half((unsigned short)h_lo))), 0u, false);
                uint32_t c_hi = e5m2_from_f32_bits<false>(
                    f2u(__half2float(__ushort_as_half((unsigned short)h_hi))), 0u, false);
                w8[j >> 1] |= (c_lo | (c_hi << 8)) << (16 * (j & 1));
            }
        }
        u32x4 oa = {ww[0], ww[1], ww[2], ww[3]}, ob = {ww[4], ww[5], ww[6], ww[7]};
        wp[0] = oa;
        wp[1] = ob;
        if constexpr (kW8) {
            u32x4 o8 = {w8[0], w8[1], w8[2], w8[3]};
            *reinterpret_cast<u32x4 *>(w8_out + g * 16) = o8;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 16) {  // ragged tail
        int64_t i = (ngroups << 4) + threadIdx.x;
        if (i < n) {
            uint32_t gc = g8[i];
            if constexpr (kStats) nonfinite += ((gc & 0x7Cu) == 0x7Cu) ? 1u : 0u;
            if (!skipping) {
                uint32_t r16 = 0;
                if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
                uint32_t h = update_one<kSR>(w16[i], gc, neg_lr, inv_scale, r16);
                w16[i] = (uint16_t)h;
                if constexpr (kW8)
                    w8_out[i] = (uint8_t)e5m2_from_f32_bits<false>(
                        f2u(__half2float(__ushort_as_half((unsigned short)h))), 0u, false);
            }
        }
    }
    if constexpr (kStats) {
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) nonfinite += __shfl_xor(nonfinite, o);
        if ((threadIdx.x & (kWave - 1)) == 0 && nonfinite) atomicAdd(&stats->nonfinite, nonfinite);
    }
}

}  // namespace mp8

extern "C" mp8_status mp8_sgd_update_fp16_sr(uint16_t *w16, const uint8_t *g8, int64_t n,
                                             float lr, float inv_loss_scale, mp8_round round,
                                             uint64_t seed, uint64_t offset,
                                             const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                             mp8_stats *stats, void *stream) {
    using namespace mp8;
    if (n < 0) return MP8_ERR_INVALID_ARG;
    if (round != MP8_RNE && round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (n == 0) return MP8_OK;
    if (!w16 || !g8) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)g8 | (uintptr_t)w8_out) & 15u) return MP8_ERR_ALIGNMENT;
    int64_t blocks = ((n >> 4) + 1 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    const float neg_lr = -lr;
    hipStream_t s = (hipStream_t)stream;
#define MP8_U(SR, W8, ST)                                                                       \
    hipLaunchKernelGGL((sgd_update_kernel<SR, W8, ST>), dim3((unsigned)blocks), dim3(256), 0, s, \
                       w16, g8, n, neg_lr, inv_loss_scale, seed, offset, skip_if_nonzero,       \
                       w8_out, stats)
    const bool sr = round == MP8_SR, w8 = w8_out != nullptr, st = stats != nullptr;
    if (sr) {
        if (w8) { if (st) MP8_U(true, true, true); else MP8_U(true, true, false); }
        else    { if (st) MP8_U(true, false, true); else MP8_U(true, false, false); }
    } else {
        if (w8) { if (st) MP8_U(false, true, true); else MP8_U(false, true, false); }
        else    { if (st) MP8_U(false, false, true); else MP8_U(false, false, false); }
    }
#undef MP8_U
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}
