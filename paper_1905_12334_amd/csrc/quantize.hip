// mp8_quantize_e5m2 / mp8_sr_bits: the Q node of Figure 1a (arXiv 1905.12334, Section 3)
// as HBM-streaming kernels for gfx950.
//
// Flat kernel: a block owns a contiguous run of the tensor; its threads read it as
// wave-interleaved 16-byte loads (every load instruction of a wave covers 1 KiB of
// contiguous FP32), convert four values to one packed dword with the hardware conversion
// instructions and store dwords (256 B contiguous per wave instruction).
// Transposing kernels: a square tile; the row-major copy is written straight from registers,
// the codes also go to an LDS tile from which the threads gather 4x4 byte blocks, transpose
// them in registers and write the transposed copy in whole 128-byte lines (tiles of 128; tiles
// of 64 only for tensors so small that latency, not traffic, sets the time).
// Shapes that are not multiples of 4 in both dimensions take a small generic kernel.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "mp8_device.hpp"

namespace mp8 {

template <bool kF16>
__device__ __forceinline__ float load_src(const void *src, int64_t i) {
    if constexpr (kF16)
        return __half2float(reinterpret_cast<const __half *>(src)[i]);
    else
        return reinterpret_cast<const float *>(src)[i];
}

// Four consecutive source elements starting at element index i (i % 4 == 0).
template <bool kF16>
__device__ __forceinline__ void load4(const void *src, int64_t i, float v[4]) {
    if constexpr (kF16) {
        u32x2 raw = __builtin_nontemporal_load(
            reinterpret_cast<const u32x2 *>(reinterpret_cast<const __half *>(src) + i));
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
        float2 a = __half22float2(h[0]), b = __half22float2(h[1]);
        v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
    } else {
        f32x4 x = __builtin_nontemporal_load(
            reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(src) + i));
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
}

// Scale and round four consecutive elements whose first has linear index i (i % 4 == 0).
template <bool kSR, bool kStats>
__device__ __forceinline__ uint32_t round4(float v[4], float scale, bool sat, const Philox &rng,
                                           int64_t i, StatsAcc &st) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] *= scale;
    uint32_t r01 = 0, r23 = 0;
    if constexpr (kSR) {
        // elements i..i+3 are halfwords (i % 8) .. +3 of Philox block i / 8
        uint4 w = rng.block((uint64_t)i >> 3);
        r01 = (i & 4) ? w.z : w.x;
        r23 = (i & 4) ? w.w : w.y;
    }
    uint32_t pk = e5m2_pack4<kSR>(v, r01, r23, sat);
    if constexpr (kStats) st.add4(v, pk);
    return pk;
}

template <bool kSR, bool kStats>
__device__ __forceinline__ uint32_t round1(float x, float scale, bool sat, const Philox &rng,
                                           int64_t i, StatsAcc &st) {
    float y = x * scale;
    uint32_t r16 = 0;
    if constexpr (kSR) r16 = philox_half(rng.block((uint64_t)i >> 3), (int)(i & 7));
    uint32_t c = e5m2_from_f32_bits<kSR>(f2u(y), r16, sat);
    if constexpr (kStats) st.add1(y, c);
    return c;
}

constexpr int kFlatUnroll = 4;  // 16-byte loads in flight per thread
constexpr int kStatsBlocks = 512;      // grid limit of the variants that end in atomics
// The flat variant with statistics: one workgroup of 1024 threads per CU.  Every workgroup ends with
// up to three atomics on the one mp8_stats, which the memory side serialises at about 17 ns each
// (measured: 2048 workgroups 142 us, 512 64 us, 256 57 us for the 67 M elements of the
// Transformer-big error tensor, against 52 us without statistics).
constexpr int kFlatStatsBlocks = 256;
constexpr int kStatsThreads = 1024;

// The flat loop of one tensor for workgroup `block` of `nblocks` (NT threads each).
template <bool kF16, bool kSR, bool kStats, int NT, int U = kFlatUnroll>
__device__ __forceinline__ void flat_body(const void *__restrict__ src, uint8_t *__restrict__ dst,
                                          int64_t n, float scale, int sat, uint64_t seed,
                                          uint64_t offset, mp8_stats *stats, int64_t block,
                                          int64_t nblocks) {
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t n4 = n >> 2;  // groups of four elements
    uint32_t *dst4 = reinterpret_cast<uint32_t *>(dst);
    const int64_t stride = nblocks * NT * U;
    for (int64_t base = block * NT * U + threadIdx.x; base < n4; base += stride) {
        float v[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = base + u * NT;
            if (g < n4) load4<kF16>(src, g * 4, v[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = base + u * NT;
            if (g < n4) {
                uint32_t pk = round4<kSR, kStats>(v[u], scale, sat != 0, rng, g * 4, st);
                // a plain store: the codes are what the next kernel (a GEMM) reads, and they are a
                // quarter of the bytes -- left in the caches they were measured 7 % faster here and
                // 11 us per step faster for the GEMM that follows than with a non-temporal store
                dst4[g] = pk;
            }
        }
    }
    // ragged tail (< 4 elements)
    if (block == 0 && threadIdx.x < 4) {
        const int64_t i = (n4 << 2) + threadIdx.x;
        if (i < n)
            dst[i] = (uint8_t)round1<kSR, kStats>(load_src<kF16>(src, i), scale, sat != 0, rng, i, st);
    }
    if constexpr (kStats) st.flush(stats);
}

template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(kStats ? kStatsThreads : 256) void quantize_flat_kernel(const void *__restrict__ src,
                                                            uint8_t *__restrict__ dst, int64_t n,
                                                            float scale, int sat, uint64_t seed,
                                                            uint64_t offset, mp8_stats *stats) {
    // the stats variant runs few, large blocks
    flat_body<kF16, kSR, kStats, kStats ? kStatsThreads : 256>(src, dst, n, scale, sat, seed, offset, stats,
                                                      blockIdx.x, gridDim.x);
}

// Several tensors in one launch: a step that quantises activations and errors (and whatever
// else is due) pays one launch, and the short tensors' start-up and tail hide behind the long
// ones' streaming.  Workgroups [first[k], first[k+1]) belong to tensor k.
constexpr int kBatchMax = 8;
struct BatchItem {
    const void *src;
    uint8_t *dst;
    int64_t n;
    float scale;
    int f16, sr, sat;
    uint64_t seed, offset;
    mp8_stats *stats;
};
struct BatchArgs {
    BatchItem item[kBatchMax];
    unsigned int first[kBatchMax + 1];
    int count;
};

__global__ __launch_bounds__(256) void quantize_batch_kernel(const BatchArgs b) {
    int k = 0;
#pragma unroll
    for (int i = 1; i < kBatchMax; ++i)
        if (i < b.count && blockIdx.x >= b.first[i]) k = i;
    k = __builtin_amdgcn_readfirstlane(k);
    // a copy of the one descriptor in scalar registers (constant indices only)
    BatchItem it = b.item[0];
#pragma unroll
    for (int i = 1; i < kBatchMax; ++i)
        if (k == i) it = b.item[i];
    unsigned int lo = b.first[0], hi = b.first[1];
#pragma unroll
    for (int i = 1; i < kBatchMax; ++i)
        if (k == i) { lo = b.first[i]; hi = b.first[i + 1]; }
    const int64_t block = blockIdx.x - lo, nblocks = hi - lo;
#define MP8_B(F16, SR, ST) \
    flat_body<F16, SR, ST, 256>(it.src, it.dst, it.n, it.scale, it.sat, it.seed, it.offset, it.stats, block, nblocks)
    const bool st = it.stats != nullptr;
    if (it.f16) {
        if (it.sr) { if (st) MP8_B(true, true, true); else MP8_B(true, true, false); }
        else       { if (st) MP8_B(true, false, true); else MP8_B(true, false, false); }
    } else {
        if (it.sr) { if (st) MP8_B(false, true, true); else MP8_B(false, true, false); }
        else       { if (st) MP8_B(false, false, true); else MP8_B(false, false, false); }
    }
#undef MP8_B
}

// Transpose a 4x4 byte block held as four row dwords into four column dwords
// (byte k of row j becomes byte j of column k).  v_perm_b32 picks bytes 0-3 from its second
// operand and 4-7 from its first.
__device__ __forceinline__ void transpose4x4(const uint32_t r[4], uint32_t c[4]) {
    const uint32_t t0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);  // r0.0 r1.0 r0.1 r1.1
    const uint32_t t1 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);  // r2.0 r3.0 r2.1 r3.1
    const uint32_t t2 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);  // r0.2 r1.2 r0.3 r1.3
    const uint32_t t3 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);  // r2.2 r3.2 r2.3 r3.3
    c[0] = __builtin_amdgcn_perm(t1, t0, 0x05040100u);
    c[1] = __builtin_amdgcn_perm(t1, t0, 0x07060302u);
    c[2] = __builtin_amdgcn_perm(t3, t2, 0x05040100u);
    c[3] = __builtin_amdgcn_perm(t3, t2, 0x07060302u);
}

constexpr int kTile = 128;
constexpr int kPitch = kTile / 4 + 1;  // LDS row pitch in dwords

// Streaming transposing kernel for large tensors: 128x128 tiles, 256 threads, and every block
// walks over several tiles (tile = blockIdx.x + i * gridDim.x).  The sixteen 16-byte loads of
// a thread's share of the NEXT tile are issued before the block turns to the transposed
// stores of the current one, so reads, row-major stores and transposed stores overlap inside
// a block instead of running in lock-step phases across the whole chip.  Phase 1: convert,
// store the row-major copy from registers, park the codes in one of two LDS tiles (pitch 33
// dwords).  Phase 2: every thread gathers 16 rows x 4 columns, transposes 4x4 byte blocks in
// registers and writes 16-byte pieces of the transposed copy, eight lanes side by side per
// 128-byte line.  Requires cols % 4 == 0 and rows % 16 == 0.
template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(256, 2) void quantize_transpose_kernel(
    const void *__restrict__ src, uint8_t *__restrict__ dst, uint8_t *__restrict__ dst_t,
    int64_t rows, int64_t cols, float scale, int sat, uint64_t seed, uint64_t offset,
    mp8_stats *stats) {
    __shared__ uint32_t tiles[2][kTile * kPitch];
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t tiles_c = (cols + kTile - 1) / kTile;
    const int64_t ntiles = ((rows + kTile - 1) / kTile) * tiles_c;
    const int tid = threadIdx.x;
    const int cq = tid & 31, tr0 = tid >> 5;   // phase 1: column group, first row (then +8)
    const int k = tid & 7, cg = tid >> 3;      // phase 2: row chunk of 16, column group
    float v[16][4];
    // Tiles that lie completely inside the tensor take code without any per-element guard:
    // with guards the compiler can no longer count outstanding loads and stores and falls
    // back to waiting for everything before each use, which serialises the stores.
    auto is_full = [&](int64_t t) {
        return (t / tiles_c + 1) * kTile <= rows && (t % tiles_c + 1) * kTile <= cols;
    };
    auto load_tile = [&](int64_t t, auto guard) {
        const int64_t r0 = (t / tiles_c) * kTile, c = (t % tiles_c) * kTile + 4 * cq;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int64_t r = r0 + tr0 + 8 * u;
            if (!decltype(guard)::value || (r < rows && c < cols)) load4<kF16>(src, r * cols + c, v[u]);
        }
    };
    auto phase1 = [&](int64_t t, uint32_t *tile, auto guard) {
        const int64_t r0 = (t / tiles_c) * kTile, c = (t % tiles_c) * kTile + 4 * cq;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int tr = tr0 + 8 * u;
            const int64_t r = r0 + tr;
            uint32_t pk = 0;
            if (!decltype(guard)::value || (r < rows && c < cols)) {
                const int64_t i = r * cols + c;
                pk = round4<kSR, kStats>(v[u], scale, sat != 0, rng, i, st);
                __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(dst + i));
            }
            tile[tr * kPitch + cq] = pk;
        }
    };
    auto phase2 = [&](int64_t t, const uint32_t *tile, auto guard) {
        const int64_t r0 = (t / tiles_c) * kTile, c0 = (t % tiles_c) * kTile;
        uint32_t colw[4][4];  // [column][row block of 4]
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            uint32_t rr[4], cc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) rr[j] = tile[(16 * k + 4 * b + j) * kPitch + cg];
            transpose4x4(rr, cc);
#pragma unroll
            for (int col = 0; col < 4; ++col) colw[col][b] = cc[col];
        }
        const int64_t orow = r0 + 16 * k;
        if (!decltype(guard)::value || orow < rows) {
#pragma unroll
            for (int col = 0; col < 4; ++col) {
                const int64_t oc = c0 + 4 * cg + col;
                if (!decltype(guard)::value || oc < cols) {
                    u32x4 o = {colw[col][0], colw[col][1], colw[col][2], colw[col][3]};
                    __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(dst_t + oc * rows + orow));
                }
            }
        }
    };
    using Guarded = std::true_type;
    using Plain = std::false_type;
    int64_t t = blockIdx.x;
    if (t < ntiles) {
        if (is_full(t)) load_tile(t, Plain{}); else load_tile(t, Guarded{});
    }
    for (int buf = 0; t < ntiles; t += gridDim.x, buf ^= 1) {
        uint32_t *tile = tiles[buf];
        const bool full = is_full(t);
        if (full) phase1(t, tile, Plain{}); else phase1(t, tile, Guarded{});
        const int64_t tn = t + gridDim.x;
        if (tn < ntiles) {
            if (is_full(tn)) load_tile(tn, Plain{}); else load_tile(tn, Guarded{});
        }
        // LDS-only synchronisation (the prefetch just issued must stay in flight); one barrier
        // per tile is enough: the other LDS tile was last read before the previous barrier
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (full) phase2(t, tile, Plain{}); else phase2(t, tile, Guarded{});
    }
    if constexpr (kStats) st.flush(stats);
}

// One tile per block (no tile loop): with thousands of tiles many blocks per CU are resident at
// different phases and this simple form streams best.  Same tile layout and phases as the
// kernel above.  Requires cols % 4 == 0 and rows % 16 == 0; not used with statistics (one
// atomic per field and block would be too many).
template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(256) void quantize_transpose_oneshot_kernel(
    const void *__restrict__ src, uint8_t *__restrict__ dst, uint8_t *__restrict__ dst_t,
    int64_t rows, int64_t cols, float scale, int sat, uint64_t seed, uint64_t offset,
    mp8_stats *stats) {
    __shared__ uint32_t tile[kTile * kPitch];
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t tiles_c = (cols + kTile - 1) / kTile;
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * kTile;
    const int64_t c0 = (int64_t)(blockIdx.x % tiles_c) * kTile;
    // phase 1: 128 rows x 32 column groups of four; item = u * 256 + tid -> (row, group)
#pragma unroll 4
    for (int u = 0; u < 16; ++u) {
        const int item = u * 256 + threadIdx.x;
        const int tr = item >> 5, cq = item & 31;
        const int64_t r = r0 + tr, c = c0 + 4 * cq;
        uint32_t pk = 0;
        if (r < rows && c < cols) {
            float v[4];
            const int64_t i = r * cols + c;
            load4<kF16>(src, i, v);
            pk = round4<kSR, kStats>(v, scale, sat != 0, rng, i, st);
            *reinterpret_cast<uint32_t *>(dst + i) = pk;
        }
        tile[tr * kPitch + cq] = pk;
    }
    __syncthreads();
    // phase 2: thread = (column group cg, row chunk k): 16 rows x 4 columns, k fastest so that
    // eight neighbouring lanes complete one 128-byte line of a transposed row
    const int k = threadIdx.x & 7, cg = threadIdx.x >> 3;
    uint32_t colw[4][4];  // [column][row block of 4]
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        uint32_t rr[4], cc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rr[j] = tile[(16 * k + 4 * b + j) * kPitch + cg];
        transpose4x4(rr, cc);
#pragma unroll
        for (int col = 0; col < 4; ++col) colw[col][b] = cc[col];
    }
    const int64_t orow = r0 + 16 * k;
    if (orow < rows) {
#pragma unroll
        for (int col = 0; col < 4; ++col) {
            const int64_t oc = c0 + 4 * cg + col;
            if (oc < cols) {
                u32x4 o = {colw[col][0], colw[col][1], colw[col][2], colw[col][3]};
                *reinterpret_cast<u32x4 *>(dst_t + oc * rows + orow) = o;
            }
        }
    }
    if constexpr (kStats) st.flush(stats);
}

// Transposing kernel, tile T x T with (T/4)^2 threads.  Phase 1: every thread converts four
// groups of four consecutive elements (a wave instruction reads whole rows of the tile), stores
// the row-major copy from registers and parks the packed codes in an LDS tile.  Phase 2: every
// thread takes one 4x4 block of bytes from LDS, transposes it in registers and stores four
// dwords of the transposed copy; T/4 neighbouring lanes complete T contiguous bytes of a
// transposed row.  Requires cols % 4 == 0 and rows % 4 == 0.  Blocks stride over the tiles,
// which are numbered super-tile by super-tile (S x S tiles each, row-major inside).
template <int T, bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__((T / 4) * (T / 4)) void quantize_tile_kernel(
    const void *__restrict__ src, uint8_t *__restrict__ dst, uint8_t *__restrict__ dst_t,
    int64_t rows, int64_t cols, float scale, int sat, uint64_t seed, uint64_t offset,
    mp8_stats *stats, int S) {
    constexpr int G = T / 4;       // column groups per tile row = threads per tile row
    constexpr int NT = G * G;      // threads
    constexpr int P = G + 1;       // LDS row pitch in dwords
    __shared__ uint32_t tile[T * P];
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t tiles_c = (cols + T - 1) / T, tiles_r = (rows + T - 1) / T;
    const int64_t sup_c = (tiles_c + S - 1) / S, sup_r = (tiles_r + S - 1) / S;
    const int64_t ntiles = sup_c * sup_r * S * S;
    const int tid = threadIdx.x;
    const int k = tid % G, cg = tid / G;  // phase 2: rows 4k..4k+3, columns 4cg..4cg+3
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t sup = t / (S * S), in = t % (S * S);
        const int64_t tr_ = (sup / sup_c) * S + in / S, tc_ = (sup % sup_c) * S + in % S;
        if (tr_ >= tiles_r || tc_ >= tiles_c) continue;
        const int64_t r0 = tr_ * T, c0 = tc_ * T;
        float v[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int item = u * NT + tid;
            const int64_t r = r0 + item / G, c = c0 + 4 * (item % G);
            if (r < rows && c < cols) load4<kF16>(src, r * cols + c, v[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int item = u * NT + tid;
            const int tr = item / G, cq = item % G;
            const int64_t r = r0 + tr, c = c0 + 4 * cq;
            uint32_t pk = 0;
            if (r < rows && c < cols) {
                const int64_t i = r * cols + c;
                pk = round4<kSR, kStats>(v[u], scale, sat != 0, rng, i, st);
                __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(dst + i));
            }
            tile[tr * P + cq] = pk;
        }
        __syncthreads();
        uint32_t rr[4], cc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rr[j] = tile[(4 * k + j) * P + cg];
        transpose4x4(rr, cc);
        const int64_t orow = r0 + 4 * k;
        if (orow < rows) {
#pragma unroll
            for (int col = 0; col < 4; ++col) {
                const int64_t oc = c0 + 4 * cg + col;
                if (oc < cols)
                    __builtin_nontemporal_store(cc[col],
                                                reinterpret_cast<uint32_t *>(dst_t + oc * rows + orow));
            }
        }
        __syncthreads();  // the tile is rewritten by the next iteration
    }
    if constexpr (kStats) st.flush(stats);
}

// Any shape: one element per thread and iteration.
template <bool kF16, bool kSR, bool kStats>
__global__ __launch_bounds__(256) void quantize_generic_kernel(
    const void *__restrict__ src, uint8_t *__restrict__ dst, uint8_t *__restrict__ dst_t,
    int64_t rows, int64_t cols, float scale, int sat, uint64_t seed, uint64_t offset,
    mp8_stats *stats) {
    const Philox rng(seed, offset);
    StatsAcc st;
    const int64_t n = rows * cols;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t c = round1<kSR, kStats>(load_src<kF16>(src, i), scale, sat != 0, rng, i, st);
        dst[i] = (uint8_t)c;
        if (dst_t != nullptr) {
            const int64_t r = i / cols;
            dst_t[(i - r * cols) * rows + r] = (uint8_t)c;
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
        // Every block of a stats variant ends with atomics on the one mp8_stats; they are
        // serialised at the memory side, so those variants run at most two 1024-thread blocks
        // per CU and stride over the tensor.
        const int nt = kStats ? kStatsThreads : 256;
        const int64_t per_block = (int64_t)nt * kFlatUnroll;
        int64_t blocks = ((n >> 2) + per_block - 1) / per_block;
        if (blocks < 1) blocks = 1;
        if (blocks > (1 << 22)) blocks = 1 << 22;  // grid-stride beyond 2^34 elements
        if (kStats && blocks > kFlatStatsBlocks) blocks = kFlatStatsBlocks;
        hipLaunchKernelGGL((quantize_flat_kernel<kF16, kSR, kStats>), dim3((unsigned)blocks),
                           dim3(nt), 0, s, src, dst, n, scale, sat, seed, offset, stats);
    } else if ((cols & 3) == 0 && (rows & 3) == 0) {
        const int64_t tr128 = (rows + 127) / 128, tc128 = (cols + 127) / 128;
        const int64_t nt = tr128 * tc128;
        const bool wide = tr128 >= 64 && tc128 >= 64;
        if (!kStats && !wide && (rows & 15) == 0 && nt >= 6144) {
            // several rounds of blocks: plain one-tile blocks, many per CU
            hipLaunchKernelGGL((quantize_transpose_oneshot_kernel<kF16, kSR, kStats>),
                               dim3((unsigned)nt), dim3(256), 0, s, src, dst, dst_t, rows, cols,
                               scale, sat, seed, offset, stats);
        } else if (!wide && (rows & 15) == 0 && nt >= 1024) {
            // a few tiles per CU: about two persistent blocks per CU, the same number of tiles
            // each, prefetching across tiles
            const int64_t per = (nt + 511) / 512;
            const int64_t blocks = (nt + per - 1) / per;
            hipLaunchKernelGGL((quantize_transpose_kernel<kF16, kSR, kStats>),
                               dim3((unsigned)blocks), dim3(256), 0, s, src, dst, dst_t, rows, cols,
                               scale, sat, seed, offset, stats);
        } else if (nt >= 64) {
            // 1024-thread blocks, all loads of a tile in flight; for a matrix that is wide in
            // both directions, super-tiles of 4x4 keep the lines written by concurrently
            // running blocks close together in both copies
            const int S = wide ? 4 : 1;
            int64_t blocks = ((tr128 + S - 1) / S) * ((tc128 + S - 1) / S) * S * S;
            if (kStats && blocks > kStatsBlocks) blocks = kStatsBlocks;
            hipLaunchKernelGGL((quantize_tile_kernel<128, kF16, kSR, kStats>),
                               dim3((unsigned)blocks), dim3(1024), 0, s, src, dst, dst_t, rows, cols,
                               scale, sat, seed, offset, stats, S);
        } else {
            // few tiles: smaller ones shorten the latency chain of the single round of blocks
            const int64_t blocks = ((rows + 63) / 64) * ((cols + 63) / 64);
            hipLaunchKernelGGL((quantize_tile_kernel<64, kF16, kSR, kStats>),
                               dim3((unsigned)blocks), dim3(256), 0, s, src, dst, dst_t, rows, cols,
                               scale, sat, seed, offset, stats, 1);
        }
    } else {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL((quantize_generic_kernel<kF16, kSR, kStats>), dim3((unsigned)blocks),
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
    if (dst_t && ((rows + kTile - 1) / kTile) * ((cols + kTile - 1) / kTile) > 0x7FFFFFFFLL)
        return MP8_ERR_UNSUPPORTED;
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

extern "C" mp8_status mp8_quantize_e5m2_batch(const mp8_quantize_item *items, int count,
                                              void *stream) {
    using namespace mp8;
    if (count < 0 || count > kBatchMax || (count > 0 && !items)) return MP8_ERR_INVALID_ARG;
    // validate everything first: on error nothing is enqueued
    for (int i = 0; i < count; ++i) {
        const mp8_quantize_item &q = items[i];
        if (q.n < 0 || (q.round != MP8_RNE && q.round != MP8_SR)) return MP8_ERR_INVALID_ARG;
        if (q.n > 0 && (!q.src || !q.dst)) return MP8_ERR_INVALID_ARG;
        if (((uintptr_t)q.src | (uintptr_t)q.dst) & 15u) return MP8_ERR_ALIGNMENT;
    }
    // Workgroups per tensor: one per 4096 elements (256 threads x 4 loads of 4 elements);
    // tensors with statistics at most kStatsBlocks, because every workgroup ends in atomics on
    // the one mp8_stats.  Tensors whose workgroups loop longest go first, so that they run
    // beside the others instead of after them.
    int order[kBatchMax];
    int64_t nblk[kBatchMax], iters[kBatchMax];
    int m = 0;
    for (int i = 0; i < count; ++i) {
        if (items[i].n == 0) continue;
        const int64_t want = ((items[i].n >> 2) + 256 * kFlatUnroll - 1) / (256 * kFlatUnroll);
        int64_t nb = std::max<int64_t>(want, 1);
        nb = std::min<int64_t>(nb, items[i].stats ? kStatsBlocks : (1 << 20));
        nblk[i] = nb;
        iters[i] = (want + nb - 1) / nb;
        order[m++] = i;
    }
    if (m == 0) return MP8_OK;
    std::stable_sort(order, order + m, [&](int x, int y) { return iters[x] > iters[y]; });
    BatchArgs args{};
    int64_t total = 0;
    for (int j = 0; j < m; ++j) {
        const mp8_quantize_item &q = items[order[j]];
        BatchItem &it = args.item[j];
        it.src = q.src;
        it.dst = q.dst;
        it.n = q.n;
        it.scale = q.scale;
        it.f16 = q.src_is_f16 != 0;
        it.sr = q.round == MP8_SR;
        it.sat = (q.flags & MP8_FLAG_SATURATE) ? 1 : 0;
        it.seed = q.seed;
        it.offset = q.offset;
        it.stats = q.stats;
        args.first[j] = (unsigned int)total;
        total += nblk[order[j]];
    }
    for (int j = m; j <= kBatchMax; ++j) args.first[j] = (unsigned int)total;
    args.count = m;
    if (total > 0x7FFFFFFFLL) return MP8_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(quantize_batch_kernel, dim3((unsigned)total), dim3(256), 0, (hipStream_t)stream, args);
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
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

// ---------------------------------------------------------------------------------------
// Measuring stick for the streaming kernels: a kernel that only moves bytes, in the access
// pattern of the flat quantize and update kernels (wave-interleaved 16-byte non-temporal loads,
// four in flight per thread) and with their read:write ratio.  What it reaches is what the
// memory system gives a kernel of this shape; the quantize and update kernels are held against it.
namespace mp8 {

// kReadsPerWrite = 4: 16 bytes read per 4 bytes written (the Q node's 4:1; the plain update's
// 3:2 sits between the two); 1: a plain copy (the optimizers with FP32 state, about 1:1).
template <int kReadsPerWrite>
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4 *__restrict__ src, void *__restrict__ dst,
                                                           int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 256 * kFlatUnroll;
    for (int64_t base = (int64_t)blockIdx.x * 256 * kFlatUnroll + threadIdx.x; base < n16; base += stride) {
        u32x4 v[kFlatUnroll];
#pragma unroll
        for (int u = 0; u < kFlatUnroll; ++u) {
            const int64_t g = base + u * 256;
            if (g < n16) v[u] = __builtin_nontemporal_load(src + g);
        }
#pragma unroll
        for (int u = 0; u < kFlatUnroll; ++u) {
            const int64_t g = base + u * 256;
            if (g < n16) {
                if constexpr (kReadsPerWrite == 4)
                    __builtin_nontemporal_store(v[u].x ^ v[u].y ^ v[u].z ^ v[u].w, reinterpret_cast<uint32_t *>(dst) + g);
                else
                    __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(dst) + g);
            }
        }
    }
}

}  // namespace mp8

extern "C" mp8_status mp8_stream_probe(const void *src, void *dst, int64_t read_bytes, int reads_per_write,
                                       void *stream) {
    if (read_bytes < 0 || (reads_per_write != 1 && reads_per_write != 4)) return MP8_ERR_INVALID_ARG;
    if (read_bytes == 0) return MP8_OK;
    if (!src || !dst) return MP8_ERR_INVALID_ARG;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15u) || (read_bytes & 15)) return MP8_ERR_ALIGNMENT;
    const int64_t n16 = read_bytes >> 4, per_block = 256 * mp8::kFlatUnroll;
    int64_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks > (1 << 22)) blocks = 1 << 22;
    if (reads_per_write == 4)
        hipLaunchKernelGGL(mp8::stream_probe_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (const mp8::u32x4 *)src, dst, n16);
    else
        hipLaunchKernelGGL(mp8::stream_probe_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (const mp8::u32x4 *)src, dst, n16);
    return hipGetLastError() == hipSuccess ? MP8_OK : MP8_ERR_HIP;
}
