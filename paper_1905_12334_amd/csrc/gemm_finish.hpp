// Second pass of a GEMM whose epilogue is not fused (split contraction, FP32 / transposed
// outputs, ragged columns), optionally with the master-weight update of Figure 1b applied to the
// codes it has just rounded; and the any-shape fallback kernel.
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

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
    // optimizer state, in place: none (plain SGD), the velocity of momentum SGD (state0), or the
    // two moments of ADAM (state0, state1) -- the rules of the stand-alone update kernels
    int states;
    float *state0, *state1;
    float mu, wd;                            // momentum; L2 regularisation of either rule
    float b1, b2, omb1, omb2, c1, c2, eps;   // ADAM
};

// One master weight from its gradient code, with the same arithmetic as the stand-alone update
// kernels; st points at this element's state words.
template <int STATES>
__device__ __forceinline__ uint32_t hook_one(const UpdateHook &u, uint32_t w16, uint32_t code, float *st,
                                             uint32_t r16) {
    if constexpr (STATES == 1) {
        const MomentumRule rule{u.neg_lr, u.mu, u.wd};
        return u.sr ? rule_one<true>(rule, w16, code, st, u.inv_scale, r16)
                    : rule_one<false>(rule, w16, code, st, u.inv_scale, 0u);
    }
    if constexpr (STATES == 2) {
        const AdamRule rule{u.neg_lr, u.b1, u.b2, u.omb1, u.omb2, u.c1, u.c2, u.eps, u.wd};
        return u.sr ? rule_one<true>(rule, w16, code, st, u.inv_scale, r16)
                    : rule_one<false>(rule, w16, code, st, u.inv_scale, 0u);
    }
    return u.sr ? update_one<true>(w16, code, u.neg_lr, u.inv_scale, r16)
                : update_one<false>(w16, code, u.neg_lr, u.inv_scale, 0u);
}

template <int STATES>
__device__ __forceinline__ void update_element(const UpdateHook &u, int64_t i, uint32_t code, uint32_t r16) {
    float st[2] = {0.0f, 0.0f};
    if constexpr (STATES >= 1) st[0] = u.state0[i];
    if constexpr (STATES == 2) st[1] = u.state1[i];
    const uint32_t h = hook_one<STATES>(u, u.w16[i], code, st, r16);
    if constexpr (STATES >= 1) u.state0[i] = st[0];
    if constexpr (STATES == 2) u.state1[i] = st[1];
    u.w16[i] = (uint16_t)h;
    if (u.w8_out != nullptr) u.w8_out[i] = (uint8_t)e5m2_of_half(h);
}

// What update4 reads of elements i0 .. i0+3: fetched before the slices are summed, so that these
// loads fly together with the slice loads instead of after them.
struct UpdateOperands4 {
    u32x2 w;
    f32x4 s0, s1;
};
template <int STATES>
__device__ __forceinline__ UpdateOperands4 load_update4(const UpdateHook &u, int64_t i0) {
    UpdateOperands4 o{};
    o.w = *reinterpret_cast<const u32x2 *>(u.w16 + i0);
    if constexpr (STATES >= 1) o.s0 = *reinterpret_cast<const f32x4 *>(u.state0 + i0);
    if constexpr (STATES == 2) o.s1 = *reinterpret_cast<const f32x4 *>(u.state1 + i0);
    return o;
}

// Elements i0 .. i0+3 (i0 % 4 == 0) from their four packed gradient codes.
template <int STATES>
__device__ __forceinline__ void update4(const UpdateHook &u, int64_t i0, uint32_t pk, const UpdateOperands4 &in) {
    uint32_t r01 = 0, r23 = 0;
    if (u.sr) {
        const Philox rng(u.seed, u.offset);
        const uint4 w = rng.block((uint64_t)i0 >> 3);
        r01 = (i0 & 4) ? w.z : w.x;
        r23 = (i0 & 4) ? w.w : w.y;
    }
    u32x2 *wp = reinterpret_cast<u32x2 *>(u.w16 + i0);
    const u32x2 wr = in.w;
    uint32_t h[4];
    const uint32_t w16v[4] = {wr.x & 0xFFFFu, wr.x >> 16, wr.y & 0xFFFFu, wr.y >> 16};
    const uint32_t r16[4] = {r01 & 0xFFFFu, r01 >> 16, r23 & 0xFFFFu, r23 >> 16};
    float st[4][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}, {0.0f, 0.0f}, {0.0f, 0.0f}};
    if constexpr (STATES >= 1) {
        const f32x4 x = in.s0;
        st[0][0] = x.x; st[1][0] = x.y; st[2][0] = x.z; st[3][0] = x.w;
    }
    if constexpr (STATES == 2) {
        const f32x4 x = in.s1;
        st[0][1] = x.x; st[1][1] = x.y; st[2][1] = x.z; st[3][1] = x.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t code = (pk >> (8 * j)) & 0xFFu;
        h[j] = hook_one<STATES>(u, w16v[j], code, st[j], r16[j]);
    }
    if constexpr (STATES >= 1) {
        const f32x4 x = {st[0][0], st[1][0], st[2][0], st[3][0]};
        *reinterpret_cast<f32x4 *>(u.state0 + i0) = x;
    }
    if constexpr (STATES == 2) {
        const f32x4 x = {st[0][1], st[1][1], st[2][1], st[3][1]};
        *reinterpret_cast<f32x4 *>(u.state1 + i0) = x;
    }
    const u32x2 o = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
    *wp = o;
    if (u.w8_out != nullptr)
        *reinterpret_cast<uint32_t *>(u.w8_out + i0) =
            e5m2_of_half(h[0]) | (e5m2_of_half(h[1]) << 8) | (e5m2_of_half(h[2]) << 16) | (e5m2_of_half(h[3]) << 24);
}

// Sum the FP32 tiles of the contraction slices in slice order and finish: the complete sum is
// rounded once.  One thread per four columns (per element when the row length is not a
// multiple of four).  STATES: state words per weight of the update rule the hook carries (0: plain
// SGD or no update at all, 1: momentum, 2: ADAM).
template <int STATES>
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
            UpdateOperands4 uo{};
            if (upd.w16 != nullptr) uo = load_update4<STATES>(upd, i0);
            // Up to eight slice loads in flight, added in slice order.  Slices beyond the last are
            // read from the last one again and replaced by +0: the running sum starts from +0 and
            // is therefore never -0, so adding +0 leaves every bit of it as it is.
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            auto add_batch = [&](int s, auto nb) {
                constexpr int NB = decltype(nb)::value;
                f32x4 x[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int sj = s + j < splits ? s + j : splits - 1;
                    x[j] = *reinterpret_cast<const f32x4 *>(partial + (int64_t)sj * slice + i0);
                }
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const bool on = s + j < splits;
                    v[0] += on ? x[j].x : 0.f; v[1] += on ? x[j].y : 0.f;
                    v[2] += on ? x[j].z : 0.f; v[3] += on ? x[j].w : 0.f;
                }
            };
            if (splits == 1) {
                add_batch(0, std::integral_constant<int, 1>{});
            } else {
                for (int s = 0; s < splits; s += 8) {
                    if (splits - s > 4) add_batch(s, std::integral_constant<int, 8>{});
                    else add_batch(s, std::integral_constant<int, 4>{});
                }
            }
            const uint32_t pk = finish4(ep, r, c, v, st);
            if (updating) update4<STATES>(upd, i0, pk, uo);
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
                update_element<STATES>(upd, i, code, r16);
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

}  // namespace mp8
