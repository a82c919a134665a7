// The general MFMA GEMM kernel (any contraction length that is a multiple of 128 bytes, every
// operand layout, the three 3x3 convolution forms).
#pragma once

#include "gemm_common.hpp"

namespace mp8 {

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
          bool BTN = false, int CONV_ = 0>
__global__ __launch_bounds__(256, MINBLOCKS) void gemm_mfma_kernel(const GemmArgs p) {
    // CONV_ 4 / 5: forms 1 / 2 for channel counts that are odd multiples of 64 (HALVES below)
    constexpr int CONV = CONV_ > 3 ? CONV_ - 3 : CONV_;
    constexpr bool HALVES = CONV_ > 3;
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
    // Convolution forms 1 and 2: stage `kstage` lies inside one tap when the contracted channel count
    // is a multiple of 128.  Otherwise (HALVES; a multiple of 64) a stage is two halves of 64
    // contraction indices ("units"), each inside one tap.  The lanes that fetch chunks 4 .. 7 of a
    // row belong to the second half; their addresses differ from the first half's by a
    // wave-uniform amount whenever the second half starts a new tap, so a stage is a uniform base
    // plus one of two non-negative offsets (`lo` for chunks 0 .. 3, `hi` for 4 .. 7) added to the
    // lane's own.  A contraction of an odd number of units ends with a stage that starts one unit
    // early: its first half repeats the stage before and is not multiplied.
    struct StageAddr {
        const uint8_t *base;
        uint32_t lo, hi;
    };
    auto first_unit = [&](int kstage, uint32_t &part) -> uint32_t {  // -> tap, part = unit within the tap
        uint32_t u = 2u * (uint32_t)(ks_begin + kstage);
        if (HALVES && p.cv.odd_units && ks_begin + kstage == p.ksteps - 1) u -= 1u;
        return fastdiv(u, p.cv.div_cpb, part);
    };
    auto a_stage = [&](int kstage) -> StageAddr {
        if constexpr (CONV == 1 || CONV == 2) {
            uint32_t part;
            const uint32_t tap = first_unit(kstage, part);
            const int s0 = CONV == 1 ? tap_shift(tap) : -tap_shift(tap);
            const int64_t b0 = (int64_t)s0 * p.lda + part * 64;
            if constexpr (!HALVES) return {a_tile + b0, 0u, 0u};
            int64_t b1 = b0;
            if ((int)part + 1 == p.cv.units_per_tap) {
                const int s1 = CONV == 1 ? tap_shift(tap + 1) : -tap_shift(tap + 1);
                b1 = (int64_t)s1 * p.lda - 64;
            }
            const int64_t least = b0 < b1 ? b0 : b1;
            return {a_tile + least, (uint32_t)(b0 - least), (uint32_t)(b1 - least)};
        } else {
            return {a_tile + (int64_t)kstage * a_kstep, 0u, 0u};
        }
    };
    auto b_stage = [&](int kstage) -> StageAddr {
        if constexpr (CONV == 2) {
            uint32_t part;
            const uint32_t tap = first_unit(kstage, part);
            const int64_t b0 = (int64_t)tap * p.cv.b_tap_stride + part * 64;
            if constexpr (!HALVES) return {b_tile + b0, 0u, 0u};
            const int64_t b1 = (int)part + 1 == p.cv.units_per_tap ? (int64_t)(tap + 1) * p.cv.b_tap_stride - 64 : b0;
            return {b_tile + b0, 0u, (uint32_t)(b1 - b0)};
        } else if constexpr (CONV == 1 && HALVES) {
            const bool early = p.cv.odd_units && ks_begin + kstage == p.ksteps - 1;
            return {b_tile + (int64_t)kstage * b_kstep - (early ? 64 * p.ldb : 0), 0u, 0u};
        } else {
            return {b_tile + (int64_t)kstage * b_kstep, 0u, 0u};
        }
    };
    const bool second_half = (lchunk & 4) != 0;   // row-major slabs: this lane fetches chunks 4 .. 7
    auto lane_off = [&](const StageAddr &sa, uint32_t own, bool halves) -> uint32_t {
        return halves ? own + (second_half ? sa.hi : sa.lo) : own;
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
        const StageAddr ak = a_stage(kstage);
        const StageAddr bk = b_stage(kstage);
#pragma unroll
        for (int q = 0; q < A_DMA; ++q) dma16(ak.base, lane_off(ak, oa[q], HALVES), sa + q * 4096);
#pragma unroll
        for (int q = 0; q < B_DMA; ++q) dma16(bk.base, lane_off(bk, ob[q], HALVES && CONV == 2), sb + q * 4096);
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
        if (q < A_DMA) {
            const StageAddr ak = a_stage(kstage);
            dma16(ak.base, lane_off(ak, oa[q < A_DMA ? q : 0], HALVES), sa + q * 4096);
        } else {
            const StageAddr bk = b_stage(kstage);
            dma16(bk.base, lane_off(bk, ob[q >= A_DMA ? q - A_DMA : 0], HALVES && CONV == 2),
                  sa + A_BYTES + (q - A_DMA) * 4096);
        }
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
    // prologue: fill the ring, fetch the fragments of (0, 0)
#pragma unroll
    for (int st = 0; st < NSTAGE; ++st)
        if (st < ks_count) issue_loads(st);
    wait_stage(-1);
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 2 * F; ++n) read_half(0, 0, frag_order(n / 2), n & 1, f0);

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
        const bool more = t + NSTAGE < ks_count;
        const bool next = t + 1 < ks_count;
        // the early stage that ends a contraction of an odd number of units: second half only
        const bool skip_first = HALVES && p.cv.odd_units && ks_begin + t == p.ksteps - 1;
#pragma unroll
        for (int k = 0; k < 2 * NM; ++k) {
            if (k < NM) {
                if (!skip_first) mfma(f0, k);
            } else {
                mfma(f1, k - NM);
            }
            if (k < S_RD) {
#pragma unroll
                for (int r = 0; r < R0; ++r) {
                    const int n = k * R0 + r;
                    if (n < 2 * F) read_half(t, 1, frag_order(n / 2), n & 1, f1);
                }
            }
            if (k == S_BAR - 1) {
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (SPLIT_BAR) wait_vm_lds<63>();  // own LDS reads only
                else wait_stage(t);
                __syncthreads();
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
    }
    wait_vm_lds<0>();

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
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if constexpr (EPI == EPI_FULL) {
        if (p.ep.stats != nullptr) st.flush(p.ep.stats);
    }
}

}  // namespace mp8
