// mp8_sgd_update_fp16_sr: the weight-update path of Figure 1b (arXiv 1905.12334, Section 3)
// as one HBM-streaming kernel for gfx950.  Per element: the 8-bit gradient is un-scaled in
// FP32, the half-precision master weight is widened to FP32, updated with one fused
// multiply-add and stored back as half with round-to-nearest-even or stochastic rounding.
// 5 bytes of traffic per element (2 + 1 read, 2 written), +1 with the optional 8-bit copy.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>

#include "mp8_device.hpp"

namespace mp8 {

constexpr int kUpdUnroll = 2;  // groups of eight elements in flight per thread

// Thread item = eight consecutive elements (16 B of weights, 8 B of gradients, one Philox
// block); items are wave-interleaved so that every load or store instruction of a wave
// covers one contiguous run.
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
    const int64_t n8 = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * 256 * kUpdUnroll;
    for (int64_t base = (int64_t)blockIdx.x * 256 * kUpdUnroll + threadIdx.x; base < n8;
         base += stride) {
        u32x2 gr[kUpdUnroll];
        u32x4 wr[kUpdUnroll];
#pragma unroll
        for (int u = 0; u < kUpdUnroll; ++u) {
            const int64_t t = base + u * 256;
            if (t < n8) {
                gr[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(g8) + t);
                if (!skipping) wr[u] = __builtin_nontemporal_load(reinterpret_cast<u32x4 *>(w16) + t);
            }
        }
#pragma unroll
        for (int u = 0; u < kUpdUnroll; ++u) {
            const int64_t t = base + u * 256;
            if (t >= n8) continue;
            const uint32_t gw[2] = {gr[u].x, gr[u].y};
            if constexpr (kStats) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    nonfinite += __builtin_popcount(((gw[q] & 0x7C7C7C7Cu) + 0x04040404u) & 0x80808080u);
            }
            if (skipping) continue;
            uint32_t ww[4] = {wr[u].x, wr[u].y, wr[u].z, wr[u].w};
            uint32_t rw[4] = {0, 0, 0, 0};
            if constexpr (kSR) {
                uint4 r = rng.block((uint64_t)t);
                rw[0] = r.x; rw[1] = r.y; rw[2] = r.z; rw[3] = r.w;
            }
            uint32_t w8[2] = {0, 0};
#pragma unroll
            for (int j = 0; j < 4; ++j) {  // pair j = elements 2j, 2j+1
                const uint32_t g_lo = (gw[j >> 1] >> (16 * (j & 1))) & 0xFFu;
                const uint32_t g_hi = (gw[j >> 1] >> (16 * (j & 1) + 8)) & 0xFFu;
                const uint32_t h_lo = update_one<kSR>(ww[j] & 0xFFFFu, g_lo, neg_lr, inv_scale, rw[j] & 0xFFFFu);
                const uint32_t h_hi = update_one<kSR>(ww[j] >> 16, g_hi, neg_lr, inv_scale, rw[j] >> 16);
                ww[j] = h_lo | (h_hi << 16);
                if constexpr (kW8)
                    w8[j >> 1] |= (e5m2_of_half(h_lo) | (e5m2_of_half(h_hi) << 8)) << (16 * (j & 1));
            }
            u32x4 o = {ww[0], ww[1], ww[2], ww[3]};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(w16) + t);
            if constexpr (kW8) {
                u32x2 o8 = {w8[0], w8[1]};
                reinterpret_cast<u32x2 *>(w8_out)[t] = o8;  // the next step's GEMM operand: stays in the caches
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 8) {  // ragged tail (< 8 elements)
        const int64_t i = (n8 << 3) + threadIdx.x;
        if (i < n) {
            const uint32_t gc = g8[i];
            if constexpr (kStats) nonfinite += ((gc & 0x7Cu) == 0x7Cu) ? 1u : 0u;
            if (!skipping) {
                uint32_t r16 = 0;
                if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
                const uint32_t h = update_one<kSR>(w16[i], gc, neg_lr, inv_scale, r16);
                w16[i] = (uint16_t)h;
                if constexpr (kW8) w8_out[i] = (uint8_t)e5m2_of_half(h);
            }
        }
    }
    if constexpr (kStats) {
        StatsAcc st;
        st.nonfinite = nonfinite;
        st.flush(stats);
    }
}

// Optimizers with state: the same item shape (eight elements) plus 32 bytes of every state
// array read and written per item; 13 bytes of traffic per element with one state array
// (momentum), 21 with two (ADAM), +1 with the 8-bit copy.
template <bool kSR, bool kW8, class Rule>
__global__ __launch_bounds__(256) void state_update_kernel(uint16_t *__restrict__ w16,
                                                           float *__restrict__ s0,
                                                           float *__restrict__ s1,
                                                           const uint8_t *__restrict__ g8, int64_t n,
                                                           const Rule rule, float inv_scale,
                                                           uint64_t seed, uint64_t offset,
                                                           const uint32_t *__restrict__ skip,
                                                           uint8_t *__restrict__ w8_out,
                                                           mp8_stats *stats) {
    constexpr int NS = Rule::kStates;
    float *const sp[2] = {s0, s1};
    const Philox rng(seed, offset);
    const bool skipping = (skip != nullptr) && (*skip != 0u);
    if (skipping && stats == nullptr) return;
    uint32_t nonfinite = 0;
    // Whole units of 512 elements, one per wave and pass: the unit is 128 chunks of four elements
    // and lane l owns chunks l and 64 + l, so that every load and store of the wave covers one
    // contiguous run (1 KB of a state array, 512 B of weights, 256 B of gradient codes) -- with
    // eight consecutive elements per lane the 16-byte accesses to the FP32 state would be strided
    // by 32 bytes and every line would be touched by two instructions.  A chunk is half a Philox
    // block; the two lanes of a pair need the same two blocks (one per chunk), each computes one
    // and hands the other lane its half.
    const int lane = threadIdx.x & 63;
    const int64_t units = n >> 9;
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
    for (int64_t u = wave0; u < units; u += nwaves) {
        const int64_t c[2] = {u * 128 + lane, u * 128 + 64 + lane};
        uint32_t gw[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            gw[h] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(g8) + c[h]);
            nonfinite += __builtin_popcount(((gw[h] & 0x7C7C7C7Cu) + 0x04040404u) & 0x80808080u);
        }
        if (skipping) continue;
        u32x2 wr[2];
        f32x4 sr[2][NS];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            wr[h] = __builtin_nontemporal_load(reinterpret_cast<u32x2 *>(w16) + c[h]);
#pragma unroll
            for (int k = 0; k < NS; ++k)
                sr[h][k] = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(sp[k]) + c[h]);
        }
        uint32_t rw[2][2] = {{0, 0}, {0, 0}};   // [chunk][word]: 16 random bits per element
        if constexpr (kSR) {
            const bool odd = (lane & 1) != 0;
            const uint4 mine = rng.block((uint64_t)(c[odd ? 1 : 0] >> 1));
            // quad_perm [1,0,3,2]: the value of the other lane of the pair
            const uint32_t got0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? mine.x : mine.z), 0xB1, 0xF, 0xF, true);
            const uint32_t got1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? mine.y : mine.w), 0xB1, 0xF, 0xF, true);
            rw[0][0] = odd ? got0 : mine.x;     // first chunk: this lane's half of the even lane's block
            rw[0][1] = odd ? got1 : mine.y;
            rw[1][0] = odd ? mine.z : got0;     // second chunk: this lane's half of the odd lane's block
            rw[1][1] = odd ? mine.w : got1;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t ww[2] = {wr[h].x, wr[h].y};
            float sv[4][NS];
#pragma unroll
            for (int k = 0; k < NS; ++k) {
                sv[0][k] = sr[h][k].x; sv[1][k] = sr[h][k].y; sv[2][k] = sr[h][k].z; sv[3][k] = sr[h][k].w;
            }
            uint32_t w8 = 0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {  // pair j = elements 2j, 2j+1 of the chunk
                const uint32_t g_lo = (gw[h] >> (16 * j)) & 0xFFu;
                const uint32_t g_hi = (gw[h] >> (16 * j + 8)) & 0xFFu;
                const uint32_t h_lo = rule_one<kSR>(rule, ww[j] & 0xFFFFu, g_lo, sv[2 * j], inv_scale, rw[h][j] & 0xFFFFu);
                const uint32_t h_hi = rule_one<kSR>(rule, ww[j] >> 16, g_hi, sv[2 * j + 1], inv_scale, rw[h][j] >> 16);
                ww[j] = h_lo | (h_hi << 16);
                if constexpr (kW8) w8 |= (e5m2_of_half(h_lo) | (e5m2_of_half(h_hi) << 8)) << (16 * j);
            }
            const u32x2 o = {ww[0], ww[1]};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x2 *>(w16) + c[h]);
#pragma unroll
            for (int k = 0; k < NS; ++k) {
                const f32x4 a = {sv[0][k], sv[1][k], sv[2][k], sv[3][k]};
                __builtin_nontemporal_store(a, reinterpret_cast<f32x4 *>(sp[k]) + c[h]);
            }
            if constexpr (kW8)
                reinterpret_cast<uint32_t *>(w8_out)[c[h]] = w8;  // the next step's GEMM operand: stays in the caches
        }
    }
    // what is left of whole items of eight elements (fewer than 64): block 0, one item per thread
    const int64_t n8 = n >> 3;
    for (int64_t t = units * 64 + threadIdx.x; blockIdx.x == 0 && t < n8; t += 256) {
        const u32x2 gr = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(g8) + t);
        const uint32_t gw[2] = {gr.x, gr.y};
#pragma unroll
        for (int q = 0; q < 2; ++q)
            nonfinite += __builtin_popcount(((gw[q] & 0x7C7C7C7Cu) + 0x04040404u) & 0x80808080u);
        if (skipping) continue;
        const u32x4 wr = __builtin_nontemporal_load(reinterpret_cast<u32x4 *>(w16) + t);
        float sv[8][NS];  // [element][state]
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(sp[k]) + 2 * t);
            const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(sp[k]) + 2 * t + 1);
            sv[0][k] = a.x; sv[1][k] = a.y; sv[2][k] = a.z; sv[3][k] = a.w;
            sv[4][k] = b.x; sv[5][k] = b.y; sv[6][k] = b.z; sv[7][k] = b.w;
        }
        uint32_t ww[4] = {wr.x, wr.y, wr.z, wr.w};
        uint32_t rw[4] = {0, 0, 0, 0};
        if constexpr (kSR) {
            uint4 r = rng.block((uint64_t)t);
            rw[0] = r.x; rw[1] = r.y; rw[2] = r.z; rw[3] = r.w;
        }
        uint32_t w8[2] = {0, 0};
#pragma unroll
        for (int j = 0; j < 4; ++j) {  // pair j = elements 2j, 2j+1
            const uint32_t g_lo = (gw[j >> 1] >> (16 * (j & 1))) & 0xFFu;
            const uint32_t g_hi = (gw[j >> 1] >> (16 * (j & 1) + 8)) & 0xFFu;
            const uint32_t h_lo = rule_one<kSR>(rule, ww[j] & 0xFFFFu, g_lo, sv[2 * j], inv_scale, rw[j] & 0xFFFFu);
            const uint32_t h_hi = rule_one<kSR>(rule, ww[j] >> 16, g_hi, sv[2 * j + 1], inv_scale, rw[j] >> 16);
            ww[j] = h_lo | (h_hi << 16);
            if constexpr (kW8)
                w8[j >> 1] |= (e5m2_of_half(h_lo) | (e5m2_of_half(h_hi) << 8)) << (16 * (j & 1));
        }
        u32x4 o = {ww[0], ww[1], ww[2], ww[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(w16) + t);
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            const f32x4 a = {sv[0][k], sv[1][k], sv[2][k], sv[3][k]};
            const f32x4 b = {sv[4][k], sv[5][k], sv[6][k], sv[7][k]};
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4 *>(sp[k]) + 2 * t);
            __builtin_nontemporal_store(b, reinterpret_cast<f32x4 *>(sp[k]) + 2 * t + 1);
        }
        if constexpr (kW8) {
            u32x2 o8 = {w8[0], w8[1]};
            reinterpret_cast<u32x2 *>(w8_out)[t] = o8;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 8) {  // ragged tail (< 8 elements)
        const int64_t i = (n8 << 3) + threadIdx.x;
        if (i < n) {
            const uint32_t gc = g8[i];
            nonfinite += ((gc & 0x7Cu) == 0x7Cu) ? 1u : 0u;
            if (!skipping) {
                uint32_t r16 = 0;
                if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
                float st[NS];
#pragma unroll
                for (int k = 0; k < NS; ++k) st[k] = sp[k][i];
                const uint32_t h = rule_one<kSR>(rule, w16[i], gc, st, inv_scale, r16);
#pragma unroll
                for (int k = 0; k < NS; ++k) sp[k][i] = st[k];
                w16[i] = (uint16_t)h;
                if constexpr (kW8) w8_out[i] = (uint8_t)e5m2_of_half(h);
            }
        }
    }
    if (stats != nullptr) {
        StatsAcc st;
        st.nonfinite = nonfinite;
        st.flush(stats);
    }
}

// Argument checks and launch shared by the optimizers with state.
template <class Rule>
static mp8_status launch_state_update(uint16_t *w16, float *s0, float *s1, const uint8_t *g8, int64_t n,
                                      const Rule &rule, float inv_loss_scale, mp8_round round,
                                      uint64_t seed, uint64_t offset, const uint32_t *skip,
                                      uint8_t *w8_out, mp8_stats *stats, void *stream) {
    if (n < 0) return MP8_ERR_INVALID_ARG;
    if (round != MP8_RNE && round != MP8_SR) return MP8_ERR_INVALID_ARG;
    if (n == 0) return MP8_OK;
    if (!w16 || !g8 || !s0 || (Rule::kStates > 1 && !s1)) return MP8_ERR_INVALID_ARG;
    if (((uintptr_t)w16 | (uintptr_t)g8 | (uintptr_t)w8_out | (uintptr_t)s0 | (uintptr_t)s1) & 15u)
        return MP8_ERR_ALIGNMENT;
    int64_t blocks = ((n >> 3) + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > (stats != nullptr ? 2048 : (1 << 22))) blocks = stats != nullptr ? 2048 : (1 << 22);
    hipStream_t s = (hipStream_t)stream;
#define MP8_M(SR, W8)                                                                                \
    hipLaunchKernelGGL((state_update_kernel<SR, W8, Rule>), dim3((unsigned)blocks), dim3(256), 0, s, \
                       w16, s0, s1, g8, n, rule, inv_loss_scale, seed, offset, skip, w8_out, stats)
    const bool sr = round == MP8_SR, w8 = w8_out != nullptr;
    if (sr) { if (w8) MP8_M(true, true); else MP8_M(true, false); }
    else    { if (w8) MP8_M(false, true); else MP8_M(false, false); }
#undef MP8_M
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}

}  // namespace mp8

extern "C" mp8_status mp8_sgd_momentum_fp16_sr(uint16_t *w16, float *velocity, const uint8_t *g8,
                                               int64_t n, float lr, float inv_loss_scale,
                                               float momentum, float weight_decay, mp8_round round,
                                               uint64_t seed, uint64_t offset,
                                               const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                               mp8_stats *stats, void *stream) {
    const mp8::MomentumRule rule{-lr, momentum, weight_decay};
    return mp8::launch_state_update(w16, velocity, nullptr, g8, n, rule, inv_loss_scale, round, seed,
                                    offset, skip_if_nonzero, w8_out, stats, stream);
}

extern "C" mp8_status mp8_adam_fp16_sr(uint16_t *w16, float *m, float *v, const uint8_t *g8, int64_t n,
                                       float lr, float inv_loss_scale, float beta1, float beta2,
                                       float eps, float weight_decay, int64_t step, mp8_round round,
                                       uint64_t seed, uint64_t offset,
                                       const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                       mp8_stats *stats, void *stream) {
    if (step < 1) return MP8_ERR_INVALID_ARG;
    // bias corrections: the powers in double, the result as FP32
    const float c1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float c2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    const mp8::AdamRule rule{-lr, beta1, beta2, 1.0f - beta1, 1.0f - beta2, c1, c2, eps, weight_decay};
    return mp8::launch_state_update(w16, m, v, g8, n, rule, inv_loss_scale, round, seed, offset,
                                    skip_if_nonzero, w8_out, stats, stream);
}

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
    const int64_t per_block = 256 * kUpdUnroll;
    int64_t blocks = ((n >> 3) + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > (1 << 22)) blocks = 1 << 22;
    if (stats != nullptr && blocks > 256 * 8) blocks = 256 * 8;  // fewer atomics: grid-stride
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
