// Device-side building blocks shared by the mp8 kernels: bit-level conversions to the
// 8-bit (1,5,2) and half (1,5,10) formats with round-to-nearest-even or stochastic
// rounding (Section 3.2 of arXiv 1905.12334), the Philox4x32-10 stream used for the
// random bits, and wave-level reductions for the overflow / amax statistics that drive
// loss scaling (Section 3.1).  gfx950 only.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mp8.h"

namespace mp8 {

constexpr int kWave = 64;

using f32x4 = float __attribute__((ext_vector_type(4)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// ---------------------------------------------------------------------------------------
// Philox4x32-10.  The key schedule is wave-uniform, so it lives in scalar registers; each
// round is two 32x32->64 multiplies and two three-input xors per lane.
// ---------------------------------------------------------------------------------------
struct Philox {
    uint32_t k0, k1, off_lo, off_hi;
    __device__ __forceinline__ Philox(uint64_t seed, uint64_t offset)
        : k0((uint32_t)seed), k1((uint32_t)(seed >> 32)), off_lo((uint32_t)offset),
          off_hi((uint32_t)(offset >> 32)) {}

    // The four output words for the group of eight elements with index / 8 == blk.
    __device__ __forceinline__ uint4 block(uint64_t blk) const {
        uint32_t c0 = (uint32_t)blk, c1 = (uint32_t)(blk >> 32), c2 = off_lo, c3 = off_hi;
        uint32_t ka = k0, kb = k1;
#pragma unroll
        for (int r = 0; r < 10; ++r) {
            uint64_t p0 = (uint64_t)0xD2511F53u * c0;
            uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
            uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ ka;
            uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ kb;
            c1 = (uint32_t)p1;
            c3 = (uint32_t)p0;
            c0 = n0;
            c2 = n2;
            ka += 0x9E3779B9u;
            kb += 0xBB67AE85u;
        }
        return make_uint4(c0, c1, c2, c3);
    }
};

// Halfword h (0..7) of a Philox block: low half of word 0 first.
__device__ __forceinline__ uint32_t philox_half(const uint4 &w, int h) {
    uint32_t word = (h >> 1) == 0 ? w.x : (h >> 1) == 1 ? w.y : (h >> 1) == 2 ? w.z : w.w;
    return (h & 1) ? (word >> 16) : (word & 0xFFFFu);
}

// ---------------------------------------------------------------------------------------
// FP32 bit pattern -> 8-bit (1,5,2) code.
//   kSR = false: round to nearest even.  kSR = true: stochastic rounding on the magnitude,
//   r16 in [0, 65536): with F the top 16 bits of the discarded fraction, the magnitude code
//   is bumped by one iff F + r16 >= 65536.
//   NaN -> 0x7F (canonical).  Inf -> sign|0x7C.  Finite overflow -> sign|0x7C, or
//   sign|0x7B when `sat`.
// The magnitude code of a normal result is (a - (112 << 23)) >> 21 because the two formats
// differ only in exponent bias (127 vs 15) and mantissa width (23 vs 2).
// ---------------------------------------------------------------------------------------
template <bool kSR>
__device__ __forceinline__ uint32_t e5m2_from_f32_bits(uint32_t u, uint32_t r16, bool sat) {
    const uint32_t a = u & 0x7FFFFFFFu;
    const uint32_t sign = (u >> 24) & 0x80u;
    uint32_t mag;
    if (a >= 0x38800000u) {  // |y| >= 2^-14: normal in the 8-bit format (or overflow)
        uint32_t t = a - 0x38000000u;
        if constexpr (kSR) {
            uint32_t F = (t >> 5) & 0xFFFFu;
            mag = (t >> 21) + ((F + r16) >> 16);
        } else {
            mag = (t + 0x000FFFFFu + ((t >> 21) & 1u)) >> 21;
        }
    } else {  // subnormal result: count of 2^-16 quanta
        if constexpr (kSR) {
            // |y| = mant * 2^(e-150); in units of 2^-32 that is mant >> (118 - e), truncated
            uint32_t e = a >> 23;
            uint32_t mant = (a & 0x007FFFFFu) | (e ? 0x00800000u : 0u);
            e = e ? e : 1u;
            uint32_t sh = 118u - e;  // >= 6 here
            uint32_t v = sh < 32u ? (mant >> sh) : 0u;
            mag = (v >> 16) + (((v & 0xFFFFu) + r16) >> 16);
        } else {
            // adding 128.0f makes the FP32 adder round |y| to a multiple of ulp(128) = 2^-16
            // with its own round-to-nearest-even
            mag = f2u(u2f(a) + 128.0f) - 0x43000000u;
        }
    }
    if (a > 0x7F800000u) return 0x7Fu;
    if (a == 0x7F800000u) return sign | 0x7Cu;
    if (mag >= 0x7Cu) mag = sat ? 0x7Bu : 0x7Cu;
    return sign | mag;
}

// ---------------------------------------------------------------------------------------
// Hardware conversions.  v_cvt_pk_bf8_f32 (round to nearest even) and v_cvt_sr_bf8_f32 fed
// with r16 << 16 (it adds the top 21 bits of its random operand to the 21 discarded mantissa
// bits) produce exactly the codes of e5m2_from_f32_bits for every FP32 input that is not a
// NaN -- including ties, subnormal results and overflow to Inf; this was checked over all
// 2^32 inputs.  For a NaN input both instructions return a NaN code (0xFE for every payload and
// either sign, measured over all 2^24 NaN patterns) and leave the neighbouring bytes alone.  The
// canonical code 0x7F is put in its place afterwards on the packed word (kBranchFree: six integer
// operations per four values, no branch -- 0.1-0.3 us faster in the GEMM epilogues, whose code
// the compiler can then schedule freely), or groups that contain a NaN take the bit-level
// routine behind a test (cheaper where conversion competes with a stream of loads for issue
// slots: the forward GEMM that quantises its activations is 1.2 us slower without the branch).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ bool any_nan4(const float y[4]) {
    return __builtin_isunordered(y[0], y[1]) | __builtin_isunordered(y[2], y[3]);
}

// Every byte of w that is a NaN code (magnitude 0x7D .. 0x7F) becomes 0x7F, sign dropped; other
// bytes stay.  No byte of m exceeds 0x7F, so the addition does not carry between bytes.
__device__ __forceinline__ uint32_t canonical_nan_codes(uint32_t w) {
    const uint32_t m = w & 0x7F7F7F7Fu;
    const uint32_t t = ((m + 0x03030303u) >> 7) & 0x01010101u;  // 1 in the bytes that hold a NaN code
    const uint32_t mask = (t << 8) - t;                          // 0xFF in those bytes (t * 255)
    return (w & ~mask) | (mask & 0x7F7F7F7Fu);
}

// Bit-level conversion of four values (groups that contain a NaN).  Out of line on
// purpose: it is rare, and keeping it out of the callers keeps their hot code small.
static inline __device__ __noinline__ uint32_t e5m2_pack4_slow(float y0, float y1, float y2, float y3,
                                                        uint32_t r01, uint32_t r23, bool sr,
                                                        bool sat) {
    const float y[4] = {y0, y1, y2, y3};
    const uint32_t r[4] = {r01 & 0xFFFFu, r01 >> 16, r23 & 0xFFFFu, r23 >> 16};
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t c = sr ? e5m2_from_f32_bits<true>(f2u(y[j]), r[j], sat)
                              : e5m2_from_f32_bits<false>(f2u(y[j]), 0u, sat);
        w |= c << (8 * j);
    }
    return w;
}


// Saturating mode on the hardware path: every finite value beyond the largest normal ends at
// +-57344 under either rounding rule (nearest-even: (57344, 61440) rounds down, the rest would
// overflow; stochastic: the bracket is [57344, 65536) and its upper end would overflow), so
// such values are replaced by +-57344 before the conversion.  Infinities stay infinities.
__device__ __forceinline__ float saturate_finite(float y) {
    const float a = __builtin_fabsf(y);
    return (a > 57344.0f && a < __builtin_inff()) ? __builtin_copysignf(57344.0f, y) : y;
}

// Four values -> four codes packed little-endian.  r01 / r23 hold the 16 random bits of
// elements (0: low half, 1: high half) and (2, 3); ignored for RNE.
template <bool kSR, bool kBranchFree = true>
__device__ __forceinline__ uint32_t e5m2_pack4(const float y[4], uint32_t r01, uint32_t r23,
                                               bool sat) {
    if constexpr (!kBranchFree) {
        if (any_nan4(y)) return e5m2_pack4_slow(y[0], y[1], y[2], y[3], r01, r23, kSR, sat);
    }
    float z[4] = {y[0], y[1], y[2], y[3]};
    if (sat) {
#pragma unroll
        for (int j = 0; j < 4; ++j) z[j] = saturate_finite(z[j]);
    }
    int w = 0;
    if constexpr (kSR) {
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[0], (int)(r01 << 16), w, 0);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[1], (int)(r01 & 0xFFFF0000u), w, 1);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[2], (int)(r23 << 16), w, 2);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[3], (int)(r23 & 0xFFFF0000u), w, 3);
    } else {
        w = __builtin_amdgcn_cvt_pk_bf8_f32(z[0], z[1], w, false);
        w = __builtin_amdgcn_cvt_pk_bf8_f32(z[2], z[3], w, true);
    }
    if constexpr (kBranchFree) return canonical_nan_codes((uint32_t)w);
    return (uint32_t)w;
}

// The same with the rounding mode chosen at run time.
template <bool kBranchFree = true>
__device__ __forceinline__ uint32_t e5m2_pack4_rt(const float y[4], uint32_t r01, uint32_t r23,
                                                  bool sr, bool sat) {
    if constexpr (!kBranchFree) {
        if (any_nan4(y)) return e5m2_pack4_slow(y[0], y[1], y[2], y[3], r01, r23, sr, sat);
    }
    float z[4] = {y[0], y[1], y[2], y[3]};
    if (sat) {
#pragma unroll
        for (int j = 0; j < 4; ++j) z[j] = saturate_finite(z[j]);
    }
    int w = 0;
    if (sr) {
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[0], (int)(r01 << 16), w, 0);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[1], (int)(r01 & 0xFFFF0000u), w, 1);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[2], (int)(r23 << 16), w, 2);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(z[3], (int)(r23 & 0xFFFF0000u), w, 3);
    } else {
        w = __builtin_amdgcn_cvt_pk_bf8_f32(z[0], z[1], w, false);
        w = __builtin_amdgcn_cvt_pk_bf8_f32(z[2], z[3], w, true);
    }
    if constexpr (kBranchFree) return canonical_nan_codes((uint32_t)w);
    return (uint32_t)w;
}

// Exact value of an 8-bit (1,5,2) code as FP32: the code is the top byte of an IEEE half.
__device__ __forceinline__ float e5m2_to_f32(uint32_t code) {
    return __half2float(__ushort_as_half((unsigned short)(code << 8)));
}

// FP32 bit pattern -> IEEE half code, same two rounding rules (13 discarded bits for normal
// results).  NaN -> 0x7E00.  Overflow -> Inf.
template <bool kSR>
__device__ __forceinline__ uint32_t f16_from_f32_bits(uint32_t u, uint32_t r16) {
    const uint32_t a = u & 0x7FFFFFFFu;
    const uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t mag;
    if (a >= 0x38800000u) {
        uint32_t t = a - 0x38000000u;
        if constexpr (kSR) {
            uint32_t F = (t & 0x1FFFu) << 3;
            mag = (t >> 13) + ((F + r16) >> 16);
        } else {
            mag = (t + 0x00000FFFu + ((t >> 13) & 1u)) >> 13;
        }
    } else {  // subnormal half: count of 2^-24 quanta
        if constexpr (kSR) {
            // units of 2^-40: mant * 2^(e-150+40) = mant >> (110 - e); e <= 112 so the shift
            // may be negative by up to 2 bits
            uint32_t e = a >> 23;
            uint32_t mant = (a & 0x007FFFFFu) | (e ? 0x00800000u : 0u);
            e = e ? e : 1u;
            int sh = 110 - (int)e;  // >= -2
            uint32_t v = sh >= 32 ? 0u : sh >= 0 ? (mant >> sh) : (mant << (-sh));
            mag = (v >> 16) + (((v & 0xFFFFu) + r16) >> 16);
        } else {
            // 0.5f has ulp 2^-24: the adder rounds |y| to a multiple of 2^-24, ties to even
            mag = f2u(u2f(a) + 0.5f) - 0x3F000000u;
        }
    }
    if (a > 0x7F800000u) return 0x7E00u;
    if (a == 0x7F800000u) return sign | 0x7C00u;
    if (mag >= 0x7C00u) mag = 0x7C00u;
    return sign | mag;
}

// ---------------------------------------------------------------------------------------
// Statistics: per-thread partials, reduced across the wave with shuffles, then one atomic
// per wave and field.
// ---------------------------------------------------------------------------------------
struct StatsAcc {
    float amax = 0.0f;      // max |y| over non-NaN values
    uint32_t nan_seen = 0;  // any NaN among the values
    uint32_t nonfinite = 0, zero_codes = 0, zero_inputs = 0;
    // four values before rounding and their packed codes
    __device__ __forceinline__ void add4(const float y[4], uint32_t packed) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            amax = __builtin_fmaxf(amax, __builtin_fabsf(y[j]));  // ignores NaN operands
            zero_inputs += (y[j] == 0.0f) ? 1u : 0u;
        }
        nan_seen |= any_nan4(y) ? 1u : 0u;
        // bytes whose exponent field is all ones: (c & 0x7C) + 4 reaches bit 7 only then
        nonfinite += __builtin_popcount(((packed & 0x7C7C7C7Cu) + 0x04040404u) & 0x80808080u);
        // bytes whose magnitude is zero
        const uint32_t z = packed & 0x7F7F7F7Fu;
        zero_codes += 4u - __builtin_popcount(((z + 0x7F7F7F7Fu) | z) & 0x80808080u);
    }
    __device__ __forceinline__ void add1(float y, uint32_t code) {
        if (y != y) nan_seen = 1u;
        amax = __builtin_fmaxf(amax, __builtin_fabsf(y));
        zero_inputs += (y == 0.0f) ? 1u : 0u;
        nonfinite += ((code & 0x7Cu) == 0x7Cu) ? 1u : 0u;
        zero_codes += ((code & 0x7Fu) == 0u) ? 1u : 0u;
    }
    // Reduce over the wave, then over the block's waves through LDS: one atomic per field
    // and block.  Every thread of the block must call this (it contains a barrier).
    __device__ __forceinline__ void flush(mp8_stats *out) {
        __shared__ uint32_t part[3][16];
        // The running maximum at the destination, fetched early so that its latency hides
        // behind the reductions: the maximum only grows, so a block whose own maximum does not
        // exceed a value already seen there has nothing to add (the load bypasses non-coherent
        // caches; an older value only makes the test more conservative).
        uint32_t seen = 0;
        if (threadIdx.x == 0)
            seen = __hip_atomic_load(&out->amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t m = nan_seen ? 0x7FC00000u : f2u(amax);
        uint32_t nf = nonfinite, z = zero_codes - zero_inputs;
        reduce_wave(m, nf, z);
        const int wave = threadIdx.x / kWave, nwaves = (blockDim.x + kWave - 1) / kWave;
        if ((threadIdx.x & (kWave - 1)) == 0) {
            part[0][wave] = m;
            part[1][wave] = nf;
            part[2][wave] = z;
        }
        __syncthreads();
        if (wave == 0) {  // the first wave combines the (at most 16) wave results
            const int l = threadIdx.x;
            m = l < nwaves ? part[0][l] : 0u;
            nf = l < nwaves ? part[1][l] : 0u;
            z = l < nwaves ? part[2][l] : 0u;
            reduce_wave(m, nf, z);
            if (l == 0) {
                if (m > seen) atomicMax(&out->amax_bits, m);
                if (nf) atomicAdd(&out->nonfinite, nf);
                if (z) atomicAdd(&out->zeroed, z);
            }
        }
    }

    // Maximum of m and sums of nf and z over the 64 lanes, left in every lane.  Four
    // data-parallel-primitive steps combine the 16 lanes of a row (neighbour, pair, mirrored
    // half row, mirrored row); the four row results are then read as scalars.
    static __device__ __forceinline__ void reduce_wave(uint32_t &m, uint32_t &nf, uint32_t &z) {
#define MP8_DPP_STEP(ctrl)                                                                    \
    {                                                                                         \
        const uint32_t om = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, ctrl, 0xF, 0xF, true);   \
        const uint32_t onf = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)nf, ctrl, 0xF, 0xF, true); \
        const uint32_t oz = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)z, ctrl, 0xF, 0xF, true);   \
        m = om > m ? om : m;                                                                  \
        nf += onf;                                                                            \
        z += oz;                                                                              \
    }
        MP8_DPP_STEP(0xB1)   // quad_perm [1,0,3,2]
        MP8_DPP_STEP(0x4E)   // quad_perm [2,3,0,1]
        MP8_DPP_STEP(0x141)  // row_half_mirror
        MP8_DPP_STEP(0x140)  // row_mirror
#undef MP8_DPP_STEP
        uint32_t rm = 0, rnf = 0, rz = 0;
#pragma unroll
        for (int row = 0; row < 4; ++row) {
            const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)m, 16 * row);
            rm = a > rm ? a : rm;
            rnf += (uint32_t)__builtin_amdgcn_readlane((int)nf, 16 * row);
            rz += (uint32_t)__builtin_amdgcn_readlane((int)z, 16 * row);
        }
        m = rm;
        nf = rnf;
        z = rz;
    }
};

// ---------------------------------------------------------------------------------------
// One element of the master-weight update of Figure 1b (shared by the update kernels and by
// the weight-gradient finishing pass that applies the update in place).
// ---------------------------------------------------------------------------------------
// value(g8) * inv_scale, FP32 weight, one fused multiply-add, rounded to half.
template <bool kSR>
__device__ __forceinline__ uint32_t update_one(uint32_t w16, uint32_t g8, float neg_lr,
                                               float inv_scale, uint32_t r16) {
    float g = e5m2_to_f32(g8) * inv_scale;
    float w = __half2float(__ushort_as_half((unsigned short)w16));
    float wn = __builtin_fmaf(neg_lr, g, w);
    // The update is an FP32 operation whose FP32 result is then converted to half: keep the
    // compiler from merging the two into one mixed-precision instruction that rounds once.
    asm volatile("" : "+v"(wn));
    if constexpr (kSR) {
        return f16_from_f32_bits<true>(f2u(wn), r16);
    } else {
        // v_cvt_f16_f32 rounds to nearest even exactly like the bit-level routine for every
        // input that is not a NaN (checked over all 2^32 inputs); NaN is made canonical
        uint32_t h = __half_as_ushort(__float2half_rn(wn));
        return (wn != wn) ? 0x7E00u : h;
    }
}

// The 8-bit (RNE) copy of a half-precision weight: the next step's operand.
__device__ __forceinline__ uint32_t e5m2_of_half(uint32_t h) {
    return e5m2_from_f32_bits<false>(f2u(__half2float(__ushort_as_half((unsigned short)h))), 0u,
                                     false);
}

// Optimizers with FP32 state in front of the same conversion.  A rule turns the un-scaled
// gradient g, the weight w and its state words into the new FP32 weight; every operation is a
// separately rounded FP32 operation in the order written (the build forbids contraction).
//
// Momentum with the L2 regularisation gradient:   g += wd * w;  v' = mu * v + g;  w' = w - lr * v'
struct MomentumRule {
    static constexpr int kStates = 1;
    float neg_lr, mu, wd;
    __device__ __forceinline__ float operator()(float w, float g, float *st) const {
        g = __builtin_fmaf(wd, w, g);
        const float v = __builtin_fmaf(mu, st[0], g);
        st[0] = v;
        return __builtin_fmaf(neg_lr, v, w);
    }
};

// ADAM (Kingma & Ba, Algorithm 1) with the same regularisation gradient:
//   m' = b1 * m + (1 - b1) * g;  v' = b2 * v + (1 - b2) * g^2
//   w' = w - lr * (m' / c1) / (sqrt(v' / c2) + eps),   c_i = 1 - b_i^step (from the host)
// Division and square root are the correctly rounded IEEE operations (the compiler's default
// for FP32 `/` and sqrt in HIP code; the approximate intrinsics are not used).
struct AdamRule {
    static constexpr int kStates = 2;
    float neg_lr, b1, b2, omb1, omb2, c1, c2, eps, wd;
    __device__ __forceinline__ float operator()(float w, float g, float *st) const {
        g = __builtin_fmaf(wd, w, g);
        const float m = __builtin_fmaf(b1, st[0], omb1 * g);
        const float v = __builtin_fmaf(b2, st[1], omb2 * (g * g));
        st[0] = m;
        st[1] = v;
        const float mhat = m / c1, vhat = v / c2;
        const float upd = mhat / (__builtin_sqrtf(vhat) + eps);
        return __builtin_fmaf(neg_lr, upd, w);
    }
};

template <bool kSR, class Rule>
__device__ __forceinline__ uint32_t rule_one(const Rule &rule, uint32_t w16, uint32_t g8, float *st,
                                             float inv_scale, uint32_t r16) {
    const float g = e5m2_to_f32(g8) * inv_scale;
    const float w = __half2float(__ushort_as_half((unsigned short)w16));
    float wn = rule(w, g, st);
    asm volatile("" : "+v"(wn));  // keep the conversion a separate, second rounding
    if constexpr (kSR) {
        return f16_from_f32_bits<true>(f2u(wn), r16);
    } else {
        uint32_t h = __half_as_ushort(__float2half_rn(wn));
        return (wn != wn) ? 0x7E00u : h;
    }
}

}  // namespace mp8
