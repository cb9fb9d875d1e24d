// Block-scaled FP8 GEMMs  OUT[i,j] = sum_r A[i,r] B[j,r]  (Jet-RL Sec. 2.2: FProp,
// DGrad and WGrad all take this form once both operands are stored with the
// reduction axis contiguous, Table 1; operand granularities of Sec. 4.2).
//
// Every kernel here computes an output element with the chain fixed in
// jet_numerics.h: p_g = one 16x16x128 FP8 MFMA over group g (accumulator input 0),
// s_g = sa*sb, acc = fma(p_g, s_g, acc) for g ascending, bf16 RNE.  p_g does not
// depend on any other group, so kernels are free to compute the p_g of different
// groups wherever they like; only the fma chain is ordered.  That keeps a token
// row bit-identical between decode-shaped and training-shaped calls (Sec. 4.1).
#include <algorithm>
#include <mutex>

#include "jet_internal.h"
#include "jet_numerics.h"

namespace jet {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Lane-linear direct global->LDS copies (no VGPR staging): lane l's 16 (4) bytes land at
// LDS address `lds` + 16 l (4 l).  `lds` and `base` must be wave-uniform.  Written as asm
// so that the copy stays asynchronous: completion is awaited explicitly with
// JET_WAIT_VMCNT + a workgroup barrier before any wave reads the data.
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void dma16(uint32_t lds, const void* base, uint32_t voff) {
    lds = __builtin_amdgcn_readfirstlane(lds);
    base = uniform_ptr(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds), "v"(voff), "s"(base)
                 : "memory");
}
// same, LDS address = lds_base + IMM formed directly in M0 (one scalar instruction)
template <int IMM>
__device__ __forceinline__ void dma16_at(uint32_t lds_base, const void* base, uint32_t voff) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base), "n"(IMM)
                 : "memory", "scc");
}
__device__ __forceinline__ void dma4(uint32_t lds, const float* ptr) {
    lds = __builtin_amdgcn_readfirstlane(lds);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :
                 : "s"(lds), "v"(ptr)
                 : "memory");
}

// One MFMA operand fragment from LDS: the lane's two 16-byte pieces.
__device__ __forceinline__ v8i load_frag(const uint8_t* lo, const uint8_t* hi) {
    return make_frag(*reinterpret_cast<const uint4*>(lo), *reinterpret_cast<const uint4*>(hi));
}

// Hardware deals workgroup b to XCD b % 8; give every XCD a contiguous range of
// logical ids so that workgroups sharing operand tiles share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int b, int n) {
    const int x = b & 7, k = b >> 3, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + k;
}

// ------------------------------------------------------------------------
// Tile kernel.  A workgroup of WI x WJ waves owns a BM x BN output tile
// (BM = WI*TM*16, BN = WJ*TN*16); a wave owns TM x TN MFMA tiles.  Workgroups are
// persistent: each one walks a list of output tiles, and the (tile, group) pairs of
// that list form one continuous stream of steps, so the copy engine, the LDS and the
// matrix core never drain between tiles.
//
// Per step the operand tiles of one group (BM + BN rows x 128 bytes) go global->LDS
// directly as whole cache lines, swizzled so that every fragment ds_read_b128 is
// conflict-free.  S LDS stages (two; four for the 128x128 and 128x64 tiles when there is at
// most one workgroup per CU); step q lives in stage q % S and is copied S - 1 steps ahead.
//
// Pipeline of one step q, written for S = 2 (t counts the wave's MFMA tiles, row m = t / TN,
// column n = t % TN):
//   top      : the column fragments cf[0..TN), the first row fragment and the scales of
//              step q are already in registers (fetched during step q-1)
//   t < last row : MFMA stream; row fragment m+1 is fetched from stage q&1 while row m runs;
//              the scale fmas of tile t-2 run on the VALU under the MFMA of tile t
//   t = first tile of the last row : every LDS read of stage q&1 has returned.  Wait for this
//              wave's copies of step q+1, workgroup barrier.  Now stage (q+1)&1 is complete
//              and stage q&1 is free: start fetching step q+1's fragments (cf[n] right after the
//              last MFMA that uses the old cf[n]) and start copying step q+2 into stage q&1.
// The only barrier of a step therefore sits in the middle of the MFMA stream, the LDS
// latency of the next step's first fragments hides under the last row of this step,
// and every copy has about one whole step to land.
//
// LDS stage layout: [A tile BM*128][B tile BN*128][scales: 256 bytes per wave]
//   tile: 1 KB block per 8 rows, copied by one instruction that moves 8 whole 128-byte
//         lines (8 consecutive lanes = one line); fragment f (rows 16f..16f+15) = blocks 2f,
//         2f+1.  Row q (0..7) of a block keeps its eight 16-byte chunks at
//         q*128 + 16*(c ^ swz), swz = (row>>1)&7, so the 16 lanes of an MFMA fragment read
//         (rows 0..15, same chunk) hit 16 different 16-byte bank groups: measured 6.4
//         cycles per ds_read_b128 (160 B/clk/CU) against 16.4 for a plain row-major tile
//   scales: wave w's 256 B = [sa rows 32w..32w+31][sb of columns 32w..32w+31, clamped to the tile]
// BM = 32 * waves, so every wave copies 4 A blocks and one scale line per step, and 4 B blocks
// (BN = 32 * waves) or 2 (BN = 16 * waves, block scales only: the 128x64 tile for batches whose
// 128x128 tiles would occupy at most half of the CUs).
// ------------------------------------------------------------------------
template <int WI, int WJ, int TM, int TN, int S = 2>
struct TileCfg {
    static constexpr int kWaves = WI * WJ;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int BM = WI * TM * 16, BN = WJ * TN * 16;
    static constexpr int kABytes = BM * 128, kBBytes = BN * 128;
    static constexpr int kBCopies = BN / (8 * kWaves);     // 1 KB blocks of the B tile per wave and step
    static constexpr int kStageBytes = kABytes + kBBytes + kWaves * 256;   // + one 256-byte scale line per wave
    static constexpr int kStages = S;                    // LDS stages: copies run kStages - 1 steps ahead
    static constexpr int kLdsBytes = kStages * kStageBytes;
    static constexpr int kOccupancy =                    // workgroups per CU: by waves and by LDS
        (512 / kThreads) < (160 * 1024 / kLdsBytes) ? (512 / kThreads) : (160 * 1024 / kLdsBytes);
    static_assert(S >= 2 && kLdsBytes <= 160 * 1024, "stages");
    static_assert(BM == 32 * kWaves && (BN == 32 * kWaves || BN == 16 * kWaves), "copy schedule");
    static_assert(TM % 2 == 0 && TN % 4 == 0, "fragment double buffer and 64-column stores assume even TM and TN a multiple of 4");
};

// Tiles of one persistent workgroup.  The hardware deals workgroup b to XCD b % 8.  The
// logical tile ids are split into 8 contiguous ranges, one per XCD, and the workgroups of
// an XCD take the ids of their range round-robin, so that at any time the workgroups of
// an XCD work on neighbouring ids (8 tile rows x a few tile columns: shared operands,
// one L2).
struct TileList {
    int first, stride, count;   // ids first + k * stride, 0 <= k < count
};
__device__ __forceinline__ TileList tiles_of_workgroup(int b, int n_wg, int n_tiles) {
    const int x = b & 7, j = b >> 3;
    const int wgs_here = (n_wg - x + 7) >> 3;
    const int q = n_tiles >> 3, rem = n_tiles & 7;
    const int start = x * q + (x < rem ? x : rem), n_here = q + (x < rem ? 1 : 0);
    TileList t;
    t.first = start + j;
    t.stride = wgs_here;
    t.count = (j < n_here) ? (n_here - j + wgs_here - 1) / wgs_here : 0;
    return t;
}

template <int SB_MODE, int WI, int WJ, int TM, int TN, int S = 2>
__global__ __launch_bounds__(64 * WI * WJ, 512 / (64 * WI * WJ))
void gemm_tile_kernel(const uint8_t* __restrict__ A, const float* __restrict__ sa,
                      const uint8_t* __restrict__ B, const float* __restrict__ sb,
                      uint16_t* __restrict__ out, int I, int ldo, int R, int tiles_i, int tiles_j) {
    using C = TileCfg<WI, WJ, TM, TN, S>;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
    const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 15, c4 = l >> 4;
    const int G = R / kGroup;

    const TileList mine = tiles_of_workgroup(blockIdx.x, gridDim.x, tiles_i * tiles_j);
    if (mine.count == 0) return;                     // whole workgroup
    const int n_steps = mine.count * G;

    // logical id -> tile origin: bands of 8 tile rows, walked column by column
    auto tile_origin = [&](int k, int& i0, int& j0) {
        constexpr int kBand = 8;
        const int lid = mine.first + k * mine.stride;
        const int band = lid / (kBand * tiles_j);
        const int within = lid - band * (kBand * tiles_j);
        const int rows_in_band = min(kBand, tiles_i - band * kBand);
        i0 = (band * kBand + within % rows_in_band) * C::BM;
        j0 = (within / rows_in_band) * C::BN;
    };

    // ---- copy cursor: the step whose operand tiles are being copied ----
    // copy schedule of this wave: A blocks 4w..4w+3, B blocks 4w..4w+3, one scale line.
    // Block c holds tile rows 32w + 8c .. + 7; lane l copies 16 bytes of row 32w + 8c + (l>>3):
    // chunk (l&7) ^ swizzle(row), swizzle = (row>>1)&7 = (l>>4) | ((c&1)<<2).
    struct Cursor {
        const uint8_t *pa, *pb;         // operand tiles of the step: tile origin + 128 g (wave-uniform)
        const float* gs;                // this lane's scale of the step
        int k, g, rows;                 // tile in the list, group, valid A rows of the tile
    };
    const uint32_t lane_row = 32 * w + (l >> 3);
    const uint32_t lane_chunk = 16 * ((l & 7) ^ (l >> 4));
    constexpr int kBC = C::kBCopies;
    static_assert(kBC == 4 || (kBC == 2 && SB_MODE == kSbBlock), "per-column scales need 32 columns per wave");
    uint32_t offB[kBC];                 // B rows never run past the end: fixed per-lane offsets
#pragma unroll
    for (int i = 0; i < kBC; ++i)
        offB[i] = (8 * kBC * w + (l >> 3) + 8 * i) * (uint32_t)R + (lane_chunk ^ ((i & 1) * 64));
    auto cursor_at_tile = [&](int k) {
        int i0, j0;
        tile_origin(k, i0, j0);
        Cursor c;
        c.pa = static_cast<const uint8_t*>(uniform_ptr(A + (size_t)i0 * R));
        c.pb = static_cast<const uint8_t*>(uniform_ptr(B + (size_t)j0 * R));
        c.k = k;
        c.g = 0;
        c.rows = I - i0;
        if (l < 32) {
            c.gs = sa + (size_t)min(i0 + 32 * w + l, I - 1) * G;
        } else if (SB_MODE == kSbBlock) {
            c.gs = sb + (size_t)((j0 + min(32 * w + (l - 32), C::BN - 1)) >> 7) * G;
        } else {
            c.gs = sb + (size_t)(j0 + 32 * w + (l - 32)) * G;
        }
        return c;
    };
    // the step after c; past the end of the list the cursor stays on the last step (its
    // tiles are then copied again into a stage nobody reads: harmless, and branch-free)
    auto cursor_after = [&](const Cursor& c) {
        Cursor n = c;
        if (c.g + 1 < G) {
            n.g = c.g + 1;
            n.pa = c.pa + kGroup;
            n.pb = c.pb + kGroup;
            n.gs = c.gs + 1;
        } else if (c.k + 1 < mine.count) {
            n = cursor_at_tile(c.k + 1);
        }
        return n;
    };
    const uint32_t ldsw = __builtin_amdgcn_readfirstlane(lds0 + 4 * w * 1024);
    const uint32_t ldsb = __builtin_amdgcn_readfirstlane(lds0 + C::kABytes + kBC * w * 1024);
    const uint32_t ldss = __builtin_amdgcn_readfirstlane(lds0 + C::kABytes + C::kBBytes + w * 256);
    constexpr int kCopies = 4 + kBC + 1;
    // copy i of step c into the stage at LDS offset st: 4 A blocks, kBC B blocks, the scale line
    auto copy_one = [&](const Cursor& c, int i, uint32_t st) {
        const uint32_t base = ldsw + st;
        if (i < 4) {
            // rows past the end of A repeat the last valid one (their outputs are never stored)
            const uint32_t row = min(lane_row + 8 * i, (uint32_t)(c.rows - 1));
            const uint32_t off = __umul24(row, (uint32_t)R) + (lane_chunk ^ ((i & 1) * 64));
            switch (i) {
                case 0: dma16_at<0>(base, c.pa, off); break;
                case 1: dma16_at<1024>(base, c.pa, off); break;
                case 2: dma16_at<2048>(base, c.pa, off); break;
                default: dma16_at<3072>(base, c.pa, off); break;
            }
        } else if (i < 4 + kBC) {
            const uint32_t bbase = ldsb + st;
            switch (i - 4) {
                case 0: dma16_at<0>(bbase, c.pb, offB[0]); break;
                case 1: dma16_at<1024>(bbase, c.pb, offB[1]); break;
                case 2: dma16_at<2048>(bbase, c.pb, offB[kBC > 2 ? 2 : 0]); break;
                default: dma16_at<3072>(bbase, c.pb, offB[kBC > 2 ? 3 : 0]); break;
            }
        } else {
            dma4(ldss + st, c.gs);
        }
    };

    // ---- fragment addressing ----
    const int wi = w / WJ, wj = w % WJ;
    // this lane's two 16-byte pieces of a fragment (row r, chunks c4 and 4 + c4)
    const int swz = (r >> 1) & 7;
    const int frag_lo = (r >> 3) * 1024 + (r & 7) * 128 + 16 * (c4 ^ swz);
    const int frag_hi = (r >> 3) * 1024 + (r & 7) * 128 + 16 * ((4 + c4) ^ swz);
    auto row_frag = [&](int slot, int m) {
        const uint8_t* p = smem + slot * C::kStageBytes + (wi * TM + m) * 2048;
        return load_frag(p + frag_lo, p + frag_hi);
    };
    auto col_frag = [&](int slot, int n) {
        const uint8_t* p = smem + slot * C::kStageBytes + C::kABytes + (wj * TN + n) * 2048;
        return load_frag(p + frag_lo, p + frag_hi);
    };
    // scales of a step as the lane needs them: sa of its row in each of the TM row tiles and
    // the scale(s) of its columns
    // (the per-column scales of WGrad are fetched at the top of the step instead: the
    // first fma needs them two MFMAs later, and there are no registers to hold them early)
    struct RawScales {
        float a[TM];
        float b_block;
    };
    auto load_scales = [&](int slot, RawScales& s) {
        const uint8_t* sc = smem + slot * C::kStageBytes + C::kABytes + C::kBBytes;
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            const int ii = (wi * TM + m) * 16 + r;
            s.a[m] = *reinterpret_cast<const float*>(sc + (ii >> 5) * 256 + (ii & 31) * 4);
        }
        if (SB_MODE == kSbBlock) {
            const int jj = wj * TN * 16;   // the wave's columns share one 128-wide block
            s.b_block = *reinterpret_cast<const float*>(sc + (jj >> 5) * 256 + 128 + (jj & 31) * 4);
        }
    };
    auto load_col_scales = [&](int slot, v4f (&s)[TN]) {
        const uint8_t* sc = smem + slot * C::kStageBytes + C::kABytes + C::kBBytes;
#pragma unroll
        for (int n = 0; n < TN; ++n) {
            const int jj = (wj * TN + n) * 16 + 4 * c4;
            s[n] = *reinterpret_cast<const v4f*>(sc + (jj >> 5) * 256 + 128 + (jj & 31) * 4);
        }
    };

    constexpr int kTiles = TM * TN, kLag = 2;
    // The scale fmas of tile t-2 run next to the MFMA of tile t, far enough behind their own
    // MFMA that its result needs no wait.  FProp/DGrad: MFMA first, three result buffers.
    // WGrad (twice the VALU work, 16 more registers of column scales): fmas first, two buffers.
    constexpr bool kFmaFirst = (SB_MODE != kSbBlock);
    constexpr int kRing = kFmaFirst ? 2 : 3;
    constexpr int kSync = (TM - 1) * TN;                 // first tile of the last row
    constexpr int kLate = kTiles + kLag - 1 - kSync;     // copies issued after the barrier of a step
    static_assert(kLate >= 1 && kLate <= kCopies && kCopies - kLate <= kSync, "copy slots");

    // ---- prologue: step 0 into stage 0, first copies of step 1, fragments of step 0 ----
    // steps 0 .. S-2 whole, the first copies of step S-1; then wait for step 0 only
    Cursor cur = cursor_at_tile(0);
#pragma unroll
    for (int s = 0; s + 1 < S; ++s) {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) copy_one(cur, i, (uint32_t)(s * C::kStageBytes));
        cur = cursor_after(cur);
    }
#pragma unroll
    for (int i = 0; i < kLate; ++i) copy_one(cur, i, (uint32_t)((S - 1) * C::kStageBytes));
    JET_WAIT_VMCNT((S - 2) * kCopies + kLate);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    v8i cf[TN], xf[2];
    RawScales next;
#pragma unroll
    for (int n = 0; n < TN; ++n) cf[n] = col_frag(0, n);
    xf[0] = row_frag(0, 0);
    load_scales(0, next);
    // s = sa * sb of the coming step (block scales: one binary32 product per row tile), formed as
    // soon as the scales are in, so that the top of a step never waits for the LDS
    float sai_n[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) sai_n[m] = (SB_MODE == kSbBlock) ? next.a[m] * next.b_block : next.a[m];

    v4f acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    // `cur` is the cursor of step q+S-1 at the top of step q (its first copies are already issued)
    for (int q = 0, k = 0, g = 0; q < n_steps; ++q) {
        const int slot = ((S & (S - 1)) == 0) ? (q & (S - 1)) : (q % S);
        const int nslot = (slot + 1 == S) ? 0 : slot + 1, oslot = (slot == 0) ? S - 1 : slot - 1;   // steps q+1, q+S-1
        const Cursor after = cursor_after(cur);     // step q+S (all control flow of a step is here)
        const uint32_t st_this = __builtin_amdgcn_readfirstlane(slot * C::kStageBytes);
        const uint32_t st_other = __builtin_amdgcn_readfirstlane(oslot * C::kStageBytes);

        // ---- one straight-line block from here to the end of the tile loop ----
        // scales of this step: s = sa * sb, one binary32 product per (row, column scale)
        float sai[TM];
        v4f sbj[TN];
#pragma unroll
        for (int m = 0; m < TM; ++m) sai[m] = sai_n[m];
        if (SB_MODE != kSbBlock) load_col_scales(slot, sbj);

        v4f pr[kRing];
#pragma unroll
        for (int t = 0; t < kTiles + kLag; ++t) {
            auto scale_fmas = [&]() {
                if (t < kLag) return;
                const int u = t - kLag, m = u / TN, n = u % TN;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float s = (SB_MODE == kSbBlock) ? sai[m] : sai[m] * sbj[n][e];
                    acc[m][n][e] = chain(pr[u % kRing][e], s, acc[m][n][e]);
                }
            };
            if (kFmaFirst) {
                scale_fmas();
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t < kTiles) {
                const int m = t / TN, n = t % TN;
                pr[t % kRing] = group_product(cf[n], xf[m & 1]);
                // next row's fragment, fetched behind the MFMA: a fetch in front of it would be
                // included in whatever LDS wait that MFMA's operands need
                __builtin_amdgcn_sched_barrier(0);
                if (n == 0 && m + 1 < TM) xf[(m + 1) & 1] = row_frag(slot, m + 1);
            }
            if (!kFmaFirst) scale_fmas();
            __builtin_amdgcn_sched_barrier(0);
            if (t == kSync) {
                // every read of stage `slot` has returned (the MFMA above needed the last one);
                // of this wave's copies only those of steps q+2 .. q+S-1 may still be on their way
                JET_WAIT_VMCNT((S - 2) * kCopies);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                cur = after;                          // step q+S goes into stage `slot`
                xf[TM & 1] = row_frag(nslot, 0);      // TM even: the buffer the last row does not use
                load_scales(nslot, next);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t == kTiles - 1) {
                // the scales fetched after the barrier are in by now (only later fetches are still out)
#pragma unroll
                for (int m = 0; m < TM; ++m) sai_n[m] = (SB_MODE == kSbBlock) ? next.a[m] * next.b_block : next.a[m];
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t >= kSync && t < kTiles) {
                cf[t - kSync] = col_frag(nslot, t - kSync);      // its last MFMA of this step is issued
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t > kSync) {
                copy_one(cur, t - kSync - 1, st_this);   // copies 0 .. kLate-1 of step q+S
                __builtin_amdgcn_sched_barrier(0);
            } else if (t < kCopies - kLate) {
                copy_one(cur, kLate + t, st_other);   // remaining copies of step q+S-1
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (++g < G) continue;
        g = 0;

        // epilogue of tile k.  A lane holds row r, columns 4 c4 .. 4 c4 + 3 of each MFMA tile.  Two
        // row-swaps between neighbouring column tiles give every lane 8 consecutive columns
        // (16 bytes) and the four lanes of a row 64 contiguous bytes; exchanging the upper eight
        // rows of one such pair of tiles with the lower eight rows of the next pair then gives
        // every row a whole 128-byte line per store instruction (8 rows x 128 B instead of
        // 16 rows x 64 B: half as many memory transactions).
        int i0, j0;
        tile_origin(k, i0, j0);
        const bool upper = (r & 8) != 0;
#pragma unroll
        for (int m = 0; m < TM; ++m) {
#pragma unroll
            for (int n = 0; n < TN; n += 4) {
                uint32_t lo[4], hi[4];   // this lane's 16 bytes of column tiles n, n+1 and of n+2, n+3
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int nn = n + 2 * half;
                    const uint32_t a0 = bf16_pack2(acc[m][nn][0], acc[m][nn][1]);
                    const uint32_t a1 = bf16_pack2(acc[m][nn][2], acc[m][nn][3]);
                    const uint32_t b0 = bf16_pack2(acc[m][nn + 1][0], acc[m][nn + 1][1]);
                    const uint32_t b1 = bf16_pack2(acc[m][nn + 1][2], acc[m][nn + 1][3]);
                    // lanes 16-31 and 48-63 of the first operand <-> lanes 0-15 and 32-47 of the second
                    const auto s0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
                    const auto s1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
                    uint32_t* d = half ? hi : lo;
                    d[0] = s0[0]; d[1] = s1[0]; d[2] = s0[1]; d[3] = s1[1];
                    acc[m][nn] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
                    acc[m][nn + 1] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
                }
                uint4 first, second;     // rows 0-7 / rows 8-15 of the row tile, 64 columns each
                uint32_t* f = &first.x;
                uint32_t* g2 = &second.x;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // row_ror:8 swaps the two halves of every 16-lane row: lane r sees lane r ^ 8
                    const uint32_t hi_x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)hi[e], 0x128, 0xf, 0xf, true);
                    const uint32_t lo_x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo[e], 0x128, 0xf, 0xf, true);
                    f[e] = upper ? hi_x : lo[e];
                    g2[e] = upper ? hi[e] : lo_x;
                }
                const int jc = j0 + (wj * TN + n + (c4 & 1)) * 16 + (c4 >> 1) * 8 + (upper ? 32 : 0);
                const int ia = i0 + (wi * TM + m) * 16 + (r & 7);
                if (ia < I) *reinterpret_cast<uint4*>(out + (size_t)ia * ldo + jc) = first;
                if (ia + 8 < I) *reinterpret_cast<uint4*>(out + (size_t)(ia + 8) * ldo + jc) = second;
            }
        }
        ++k;
    }
    JET_WAIT_VMCNT(0);   // nothing may be in flight towards the LDS when it is released
}

// ------------------------------------------------------------------------
// Skinny kernel for I <= 32 (decode): bound by streaming B (the weights) once.
// A workgroup of kSkWaves waves owns 16 output columns and the whole reduction.  The
// groups of a pass (32 / RM groups) are dealt to the waves in runs of consecutive
// groups; every wave streams its own units (16 weight rows + the 16 or 32 activation
// rows + scales of one group) through a private LDS ring with kSkDepth units in flight,
// using the same whole-line LDS-DMA and swizzled fragment layout as the tile kernel --
// no barrier is needed for the ring.  After every pass the p_g and s_g meet in LDS and
// four waves per row tile run the ordered fma chain for their quarter of the outputs.
// ------------------------------------------------------------------------
constexpr int sk_unit_bytes(int rm) { return 2048 + rm * 2048 + 256; }    // weight fragment, RM activation fragments, scales
constexpr int sk_group_bytes(int rm) { return rm * (4 * 64 * 4 + 64 * 4); } // per row tile: p[4][64] + s[64]
constexpr int sk_pass(int rm) { return 32 / rm; }                          // groups chained per pass
constexpr int sk_lds_bytes(int depth, int waves, int rm) {
    return waves * depth * sk_unit_bytes(rm) + sk_pass(rm) * sk_group_bytes(rm);
}

// kSkDepth = units in flight per wave: 3 or 6 when there is at most one workgroup per CU, 1 when
// the strips outnumber the CUs (two workgroups then share a CU and cover each other's start-up,
// chain passes and drain)
// kSkWaves = waves splitting the groups of a strip (runs of consecutive groups): 8 unless the
// reduction is very short
// RM = 16-row tiles of the batch (1: I <= 16, 2: I <= 32); a unit then carries RM activation
// fragments and gives RM MFMAs with the same weight fragment
// ABLK = 8-row blocks of activations that hold a row of the batch ((I + 7) / 8): only these are
// copied, and of the last one only the lines of existing rows -- every byte through a CU's
// memory pipeline costs the same there whether it misses or hits, so at I = 1 the copy of 15
// repeated rows would double the time of a strip.  The fragments of the other rows are read from
// LDS that no copy wrote; their products land in output rows that are never stored.
template <int kSkDepth, int kSkWaves, int RM, int ABLK = 2 * RM>
__global__ __launch_bounds__(64 * kSkWaves) void gemm_skinny_kernel(const uint8_t* __restrict__ A,
                                                                     const float* __restrict__ sa,
                                                                     const uint8_t* __restrict__ B,
                                                                     const float* __restrict__ sb,
                                                                     uint16_t* __restrict__ out, int I, int J,
                                                                     int R) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
    const int t = threadIdx.x, w = t >> 6, l = t & 63, r = l & 15, c4 = l >> 4;
    constexpr int kUnit = sk_unit_bytes(RM), kGroupBytes = sk_group_bytes(RM), kPass = sk_pass(RM);
    constexpr int kSkRingBytes = kSkDepth * kUnit;
    constexpr int kSkRun = kPass / kSkWaves;                 // consecutive groups per wave per pass
    constexpr int kCopies = 2 + ABLK + 1;                    // vector-memory operations per unit
    static_assert(kSkRun >= 1 && RM <= 2 && 4 * RM <= kSkWaves && (kSkDepth - 1) * kCopies < 64, "");
    static_assert(ABLK >= 1 && ABLK <= 2 * RM, "");
    const int G = R / kGroup;
    const int j0 = blockIdx.x * 16;

    // copy offsets of this lane: block b = rows 8b..8b+7, one line per 8 lanes
    uint32_t offW[2], offX[ABLK];
    bool rowX[ABLK];                                         // this lane's row of block b exists
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int row = 8 * b + (l >> 3);
        offW[b] = (uint32_t)row * (uint32_t)R + 16 * ((l & 7) ^ ((row >> 1) & 7));
    }
#pragma unroll
    for (int b = 0; b < ABLK; ++b) {
        const int row = 8 * b + (l >> 3);
        rowX[b] = row < I;
        offX[b] = (uint32_t)min(row, I - 1) * (uint32_t)R + 16 * ((l & 7) ^ ((row >> 1) & 7));
    }
    const uint8_t* baseW = B + (size_t)j0 * R;
    // scale line of a unit: lanes 0 .. 16 RM - 1 fetch sa of the batch rows (clamped), lanes 32-63 the block scale
    const float* gs = (l < 32) ? sa + (size_t)min(l, I - 1) * G : sb + (size_t)(j0 >> 7) * G;
    const int swz = (r >> 1) & 7;
    const int frag_lo = (r >> 3) * 1024 + (r & 7) * 128 + 16 * (c4 ^ swz);
    const int frag_hi = (r >> 3) * 1024 + (r & 7) * 128 + 16 * ((4 + c4) ^ swz);

    const uint32_t ring = __builtin_amdgcn_readfirstlane(lds0 + w * kSkRingBytes);
    uint8_t* const ring_p = smem + w * kSkRingBytes;
    uint8_t* const pass_p = smem + kSkWaves * kSkRingBytes;

    // unit i of this wave is group seq(i); the wave has n_units of them
    auto seq = [&](int i) { return (i / kSkRun) * kPass + w * kSkRun + (i % kSkRun); };
    const int full = G / kPass, tail = G - full * kPass;
    const int n_units = full * kSkRun + max(0, min(kSkRun, tail - w * kSkRun));

    auto issue = [&](int i) {
        const int g = seq(i);
        const uint32_t u = ring + (i % kSkDepth) * kUnit;
        dma16(u, baseW + (size_t)g * kGroup, offW[0]);
        dma16(u + 1024, baseW + (size_t)g * kGroup, offW[1]);
        // (block b < ABLK always holds row 8 b < I, so every wave issues the same number of copies)
#pragma unroll
        for (int b = 0; b < ABLK; ++b)
            if (rowX[b]) dma16(u + 2048 + b * 1024, A + (size_t)g * kGroup, offX[b]);
        dma4(u + 2048 + RM * 2048, gs + g);
    };

    for (int i = 0; i < kSkDepth && i < n_units; ++i) issue(i);

    // chain owner: wave w < 4 RM owns row tile w >> 2 and the columns j0 + 4 c4 + (w & 3)
    const int cm = w >> 2, cq = w & 3;
    float acc = 0.0f;
    int i = 0;
    for (int g0 = 0; g0 < G; g0 += kPass) {
        const int ng = min(kPass, G - g0);
        for (int j = 0; j < kSkRun; ++j, ++i) {
            if (i >= n_units) break;                 // wave-uniform
            // unit i has landed once at most the younger units' copies are outstanding
            const int younger = min(n_units, i + kSkDepth) - i - 1;
            switch (younger) {
                case 0: JET_WAIT_VMCNT(0); break;
                case 1: JET_WAIT_VMCNT(kCopies); break;
                case 2: JET_WAIT_VMCNT(2 * kCopies); break;
                case 3: JET_WAIT_VMCNT(3 * kCopies); break;
                case 4: JET_WAIT_VMCNT(4 * kCopies); break;
                default: JET_WAIT_VMCNT(5 * kCopies); break;
            }
            asm volatile("" ::: "memory");
            const uint8_t* u = ring_p + (i % kSkDepth) * kUnit;
            const v8i wf = load_frag(u + frag_lo, u + frag_hi);
            const float sbv = *reinterpret_cast<const float*>(u + 2048 + RM * 2048 + 128);
            float* dst = reinterpret_cast<float*>(pass_p + (seq(i) - g0) * kGroupBytes);
#pragma unroll
            for (int m = 0; m < RM; ++m) {
                const v8i xf = load_frag(u + 2048 + m * 2048 + frag_lo, u + 2048 + m * 2048 + frag_hi);
                const float s = *reinterpret_cast<const float*>(u + 2048 + RM * 2048 + 4 * (16 * m + r)) * sbv;
                const v4f p = group_product(wf, xf);
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[m * 320 + e * 64 + l] = p[e];
                dst[m * 320 + 256 + l] = s;
            }
            asm volatile("" ::: "memory");
            if (i + kSkDepth < n_units) issue(i + kSkDepth);
        }
        __syncthreads();
        if (w < 4 * RM) {                                // wave-uniform
            const float* src = reinterpret_cast<const float*>(pass_p) + cm * 320;
            if (ng == kPass) {
                // all LDS reads of the pass first, then the ordered chain: a loop of read, read, fma
                // pays the LDS latency once per group (1.6 us per pass of 32 groups)
                float pv[kPass], sv[kPass];
#pragma unroll
                for (int g = 0; g < kPass; ++g) {
                    pv[g] = src[g * (kGroupBytes / 4) + cq * 64 + l];
                    sv[g] = src[g * (kGroupBytes / 4) + 256 + l];
                }
#pragma unroll
                for (int g = 0; g < kPass; ++g) acc = chain(pv[g], sv[g], acc);
            } else {
                for (int g = 0; g < ng; ++g)
                    acc = chain(src[g * (kGroupBytes / 4) + cq * 64 + l], src[g * (kGroupBytes / 4) + 256 + l], acc);
            }
        }
        __syncthreads();
    }
    const int row = 16 * cm + r;
    if (w < 4 * RM && row < I) out[(size_t)row * J + j0 + 4 * c4 + cq] = (uint16_t)bf16_rne(acc);
}

// ------------------------------------------------------------------------
// Strip kernel for decode batches, 16 < I <= 256 (block scales only).  The weights are
// streamed once per row block of the batch, so the kernel lives on memory-level
// parallelism, not on the matrix core.  A workgroup of 8 waves owns a (16 RM) x (16 CN)
// output tile and walks the whole reduction two groups (a "pair") at a time.  Waves 0-3
// (one per SIMD) compute; waves 4-7 only copy, so that no MFMA stream ever waits behind
// a copy.  The weight rows and scale lines (from HBM) and the activation rows
// (L2-resident) travel global->LDS through two separate rings.  The outstanding-copy
// counter of a wave retires in issue order, so a wave that issued both streams could
// never keep the weights further ahead than the activations: waves 4 and 5 copy only
// weights and scales, waves 6 and 7 only activations.  One barrier per pair; the
// fragments of pair p+2 are fetched from LDS into registers while pair p is computed, so
// neither the LDS latency nor the barrier is paid per group.  Computing wave w owns
// RM*CN/4 of the MFMA tiles and runs their ordered fma chains in registers: the same chain
// as every other kernel, so rows are bit-identical.
// Two configurations: 32-row blocks with rings shallow enough for two workgroups per CU
// (they cover each other's start-up and drain), 64-row blocks with deep rings.
// ------------------------------------------------------------------------
template <int RM, int CN, int WDEPTH, int ADEPTH>
struct StripCfg {
    static constexpr int kWaves = 4;
    static constexpr int BM = 16 * RM, BN = 16 * CN;
    static constexpr int kWDepth = WDEPTH, kADepth = ADEPTH;    // ring depths in pairs
    static constexpr int kWGroup = CN * 2048 + 512;             // weight fragments, then sa[64] and the sb line
    static constexpr int kAGroup = RM * 2048;                   // activation fragments
    static constexpr int kWStage = 2 * kWGroup, kAStage = 2 * kAGroup;
    static constexpr int kSinkBytes = 256;                      // landing zone of the L2 warm-up loads
    // 64-row blocks fetch the activation scales a chunk of 16 groups ahead, [row][16 groups], into
    // three chunk buffers (the one being read, the next one, and the one being filled); 32-row
    // blocks fetch one scale per row with every group (measured: the chunks gain 15 % on 64-row
    // blocks with a long reduction and lose 10 % on 32-row blocks with a short one)
    static constexpr bool kSaAhead = BM == 64;
    static constexpr int kSaChunk = 16, kSaBufBytes = BM * kSaChunk * 4, kSaBufs = 3;
    static constexpr int kSaOffset = kWDepth * kWStage + kADepth * kAStage + kSinkBytes;
    static constexpr int kLdsBytes = kSaOffset + (kSaAhead ? kSaBufs * kSaBufBytes : 0);
    static constexpr int kWOps = 2 * (CN + 1), kAOps = 2 * RM;  // copies per wave per pair
    static constexpr int kTiles = RM * CN / kWaves;             // MFMA tiles per wave
    static constexpr int kNM = (kTiles + CN - 1) / CN;          // distinct row tiles per wave
    static constexpr int kNN = kTiles < CN ? kTiles : CN;       // distinct column tiles per wave
    static constexpr int kFetchOps = 2 * (2 * (kNM + kNN) + kNM + 1);   // LDS reads of one pair
    static_assert(RM % 2 == 0 && CN % 2 == 0 && RM * CN % kWaves == 0 && BM <= 64 && 128 % BN == 0, "");
    static_assert(kNM * kNN == kTiles, "a wave's tiles form a kNM x kNN rectangle");
    static_assert(kWDepth >= 4 && kADepth >= 4 && (kWDepth - 3) * kWOps < 64 && (kADepth - 3) * kAOps < 64, "");
    // Iteration p fills the buffer of chunk (2 (p + kWDepth) + 1) / 16 + 1 while the reads are at group
    // 2 p + 4 or later: the chunk that buffer held (three chunks back) must be behind every read.
    static_assert(kSaChunk == 16 && BM / 4 <= kSaChunk && (!kSaAhead || 2 * kWDepth + 1 < kSaChunk + 6), "");
    static_assert(kLdsBytes <= 160 * 1024, "");
};

template <int RM, int CN, int WDEPTH, int ADEPTH>
__global__ __launch_bounds__(512) void gemm_strip_kernel(const uint8_t* __restrict__ A,
                                                          const float* __restrict__ sa,
                                                          const uint8_t* __restrict__ B,
                                                          const float* __restrict__ sb,
                                                          uint16_t* __restrict__ out, int I, int J, int R,
                                                          int row_blocks) {
    using C = StripCfg<RM, CN, WDEPTH, ADEPTH>;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
    const int t = threadIdx.x, w = __builtin_amdgcn_readfirstlane(t >> 6), l = t & 63, r = l & 15, c4 = l >> 4;
    const int G = R / kGroup, P = (G + 1) / 2;

    // workgroups that share a weight strip (different row blocks) sit next to each other on
    // one XCD, so the strip leaves HBM once
    const int strips = J / C::BN, b = blockIdx.x;
    int rb, strip;
    if (strips % 8 == 0) {
        rb = (b >> 3) % row_blocks;
        strip = ((b >> 3) / row_blocks) * 8 + (b & 7);
    } else {
        rb = b % row_blocks;
        strip = b / row_blocks;
    }
    const int i0 = rb * C::BM, j0 = strip * C::BN;

    // ---- copies: a wave copies kMine consecutive 1 KB blocks (8 rows) of each group of a
    // pair; block b is half b & 1 of fragment b >> 1 ----
    // waves 0-3 compute (one per SIMD); waves 4-7 only copy: 4, 5 the weights, 6, 7 the activations
    const bool copier = w >= 4;
    const bool w_stream = w < 6;
    const int side = w & 1;
    constexpr int kWMine = CN, kAMine = RM;
    constexpr int kMineMax = RM > CN ? RM : CN;
    const uint32_t lane_chunk = 16 * ((l & 7) ^ (l >> 4));
    const uint8_t* baseW = static_cast<const uint8_t*>(uniform_ptr(B + (size_t)j0 * R));
    const uint8_t* baseA = static_cast<const uint8_t*>(uniform_ptr(A + (size_t)i0 * R));
    uint32_t off[kMineMax];
#pragma unroll
    for (int i = 0; i < kMineMax; ++i) {
        if (w_stream) {
            const int blk = side * kWMine + (i < kWMine ? i : 0);
            off[i] = (uint32_t)(8 * blk + (l >> 3)) * (uint32_t)R + (lane_chunk ^ ((blk & 1) * 64));
        } else {
            const int blk = side * kAMine + (i < kAMine ? i : 0);
            const int row = min(i0 + 8 * blk + (l >> 3), I - 1) - i0;   // rows past the end repeat the last one
            off[i] = (uint32_t)row * (uint32_t)R + (lane_chunk ^ ((blk & 1) * 64));
        }
    }
    // scales travel with the weights (the weight waves have far fewer copies to issue than the
    // activation waves).  Wave 5 copies the block scale of every group.  Wave 4 copies the
    // activation scales: one per row with every group, or (kSaAhead) a chunk of 16 groups ahead:
    // with group g it fetches 4 rows x the 16 groups of the next chunk (4 cache lines per
    // instruction instead of one per lane), so the chunk after g's is complete before its
    // first group is.
    const bool sa_wave = w == 4;
    const float* sb_line = sb + (size_t)(j0 >> 7) * G;
    const float* gs = sa_wave ? sa + (size_t)min(i0 + l, I - 1) * G : sb_line;   // one scale per lane and group
    const int sa_grp = l & 15;
    const int sa_off0 = (i0 + (l >> 4)) * G, sa_off_last = (I - 1) * G;          // chunk copies: this lane's row of quad 0
    const uint32_t lds_w = __builtin_amdgcn_readfirstlane(lds0 + side * kWMine * 1024);
    const uint32_t lds_a = __builtin_amdgcn_readfirstlane(lds0 + C::kWDepth * C::kWStage + side * kAMine * 1024);
    const uint32_t lds_s = __builtin_amdgcn_readfirstlane(lds0 + CN * 2048 + side * 256);
    const uint32_t lds_sa = __builtin_amdgcn_readfirstlane(lds0 + C::kSaOffset);
    // rows 4 rq .. 4 rq + 3 of the tile (past the end: the last row), groups of chunk c (past the end: the last group)
    auto sa_src = [&](int c, int rq) {
        return sa + min(sa_off0 + rq * 4 * G, sa_off_last) + min(C::kSaChunk * c + sa_grp, G - 1);
    };
    auto sa_dst = [&](int c, int rq) { return lds_sa + (c % C::kSaBufs) * C::kSaBufBytes + rq * 256; };
    // this wave's copies of pair p (groups past the end repeat the last one)
    auto issue = [&](int p) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int g = min(2 * p + h, G - 1);
            if (w_stream) {
                const uint32_t st = (p % C::kWDepth) * C::kWStage + h * C::kWGroup;
#pragma unroll
                for (int i = 0; i < kWMine; ++i) dma16(lds_w + st + i * 1024, baseW + (size_t)g * kGroup, off[i]);
                // (a branch between the two waves' copies: selecting source and destination per copy
                // instead measured 10 % slower)
                if (!C::kSaAhead || !sa_wave) {
                    dma4(lds_s + st, gs + g);
                } else {
                    const int c = g / C::kSaChunk + 1, rq = (g % C::kSaChunk) % (C::BM / 4);
                    dma4(sa_dst(c, rq), sa_src(c, rq));
                }
            } else {
                const uint32_t st = (p % C::kADepth) * C::kAStage + h * C::kAGroup;
#pragma unroll
                for (int i = 0; i < kAMine; ++i) dma16(lds_a + st + i * 1024, baseA + (size_t)g * kGroup, off[i]);
            }
        }
    };

    // ---- this wave's MFMA tiles: rows m0 .. m0+kNM-1, columns n0 .. n0+kNN-1 (in tiles) ----
    const int first = (w & 3) * C::kTiles, m0 = first / CN, n0 = first % CN;
    const int swz = (r >> 1) & 7;
    const int frag_lo = (r >> 3) * 1024 + (r & 7) * 128 + 16 * (c4 ^ swz);
    const int frag_hi = (r >> 3) * 1024 + (r & 7) * 128 + 16 * ((4 + c4) ^ swz);
    struct Operands {           // of one pair
        v8i wf[2][C::kNN], xf[2][C::kNM];
        float sa[2][C::kNM], sb[2];
    };
    auto fetch = [&](int p, Operands& o) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int g = min(2 * p + h, G - 1);
            const uint8_t* ps = smem + C::kSaOffset + ((g / C::kSaChunk) % C::kSaBufs) * C::kSaBufBytes + (g % C::kSaChunk) * 4;
            const uint8_t* pw = smem + (p % C::kWDepth) * C::kWStage + h * C::kWGroup;
            const uint8_t* pa = smem + C::kWDepth * C::kWStage + (p % C::kADepth) * C::kAStage + h * C::kAGroup;
#pragma unroll
            for (int n = 0; n < C::kNN; ++n)
                o.wf[h][n] = load_frag(pw + (n0 + n) * 2048 + frag_lo, pw + (n0 + n) * 2048 + frag_hi);
#pragma unroll
            for (int m = 0; m < C::kNM; ++m) {
                o.xf[h][m] = load_frag(pa + (m0 + m) * 2048 + frag_lo, pa + (m0 + m) * 2048 + frag_hi);
                o.sa[h][m] = C::kSaAhead
                                 ? *reinterpret_cast<const float*>(ps + ((m0 + m) * 16 + r) * (C::kSaChunk * 4))
                                 : *reinterpret_cast<const float*>(pw + CN * 2048 + ((m0 + m) * 16 + r) * 4);
            }
            o.sb[h] = *reinterpret_cast<const float*>(pw + CN * 2048 + 256);
        }
    };
    v4f acc[C::kNM][C::kNN];
#pragma unroll
    for (int m = 0; m < C::kNM; ++m)
#pragma unroll
        for (int n = 0; n < C::kNN; ++n) acc[m][n] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    auto compute = [&](int p, const Operands& o) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (2 * p + h >= G) break;               // odd G: the last pair has one group
#pragma unroll
            for (int m = 0; m < C::kNM; ++m) {
                const float s = o.sa[h][m] * o.sb[h];
#pragma unroll
                for (int n = 0; n < C::kNN; ++n) {
                    const v4f pg = group_product(o.wf[h][n], o.xf[h][m]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[m][n][e] = chain(pg[e], s, acc[m][n][e]);
                }
            }
        }
    };
    // "of my copies only those of the last n pairs I issued may still be on their way", n = depth - less
    auto wait_copies = [&](int less) {
        if (w_stream) {
            if (less == 3) JET_WAIT_VMCNT((C::kWDepth - 3) * C::kWOps);
            else JET_WAIT_VMCNT((C::kWDepth - 2) * C::kWOps);
        } else {
            if (less == 3) JET_WAIT_VMCNT((C::kADepth - 3) * C::kAOps);
            else JET_WAIT_VMCNT((C::kADepth - 2) * C::kAOps);
        }
    };

    // ---- L2 warm-up of this row block's activations ----
    // Every workgroup of an XCD walks the same activation rows group by group at about the
    // same time, so without help each group's copy would be a fresh miss to HBM.  The
    // workgroups of an XCD touch one dword of every cache line once, up front, sharing the
    // lines between them; the ring copies then hit in the L2.
    {
        const int per_xcd = (gridDim.x + 7) >> 3, me = b >> 3;
        const int rows = min(C::BM, I - i0);
        const long lines = (long)rows * G;
        const uint32_t sink = __builtin_amdgcn_readfirstlane(lds0 + C::kWDepth * C::kWStage + C::kADepth * C::kAStage);
        for (long x = (long)me * 512 + t; x < lines; x += (long)per_xcd * 512) {
            const long row = x / G, g = x - row * G;
            dma4(sink, reinterpret_cast<const float*>(baseA + (size_t)row * R + (size_t)g * kGroup));
        }
    }

    // ---- prologue: fill both rings, fetch pairs 0 and 1 ----
    // iteration p of the main loop issues pair p + depth; the prologue issues pairs 0 .. depth-1
    // in the same relative order, so the steady-state counts hold from the start
    if (C::kSaAhead && !copier) {
        // chunk 0 of the activation scales: the computing waves have nothing else to do yet
        for (int rq = w; rq < C::BM / 4; rq += C::kWaves) dma4(sa_dst(0, rq), sa_src(0, rq));
        JET_WAIT_VMCNT(0);
    }
    for (int v = 0; v < C::kWDepth; ++v)
        if (copier && (w_stream || v < C::kADepth)) issue(v);
    if (copier) wait_copies(2);                      // pairs 0 and 1 landed: depth-2 later pairs outstanding
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // iteration p (one barrier): pairs <= p+2 have landed; the slots of pair p are free (its
    // fragments are in registers).  The two kinds of wave run the same number of barriers.
    // (Refilling the slots of pair p+1 as well -- one more pair in flight -- needs every LDS read of
    // an iteration to return before the next barrier; measured: a few percent faster when the weights
    // come from HBM, 10-25 % slower when they are cache-resident.)
    if (copier) {
        for (int p = 0; p < P; ++p) {
            wait_copies(3);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue(p + (w_stream ? C::kWDepth : C::kADepth));
        }
        JET_WAIT_VMCNT(0);   // nothing may be in flight towards the LDS when it is released
        return;
    }
    Operands op0, op1, op2;
    fetch(0, op0);
    fetch(min(1, P - 1), op1);
    auto iteration = [&](int p, const Operands& cur, Operands& nxt2) {
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        fetch(min(p + 2, P - 1), nxt2);
        compute(p, cur);
        // my reads of pair p+1's slots are done before the next barrier lets them be overwritten
        // (LDS reads return in order: at most the reads of pair p+2 stay outstanding)
        __builtin_amdgcn_s_waitcnt(0xc07f | ((C::kFetchOps < 15 ? C::kFetchOps : 15) << 8));
    };
    int p = 0;
    for (; p + 2 < P; p += 3) {
        iteration(p, op0, op2);
        iteration(p + 1, op1, op0);
        iteration(p + 2, op2, op1);
    }
    if (p < P) iteration(p, op0, op2);
    if (p + 1 < P) iteration(p + 1, op1, op0);
    JET_WAIT_VMCNT(0);   // nothing may be in flight towards the LDS when it is released

#pragma unroll
    for (int m = 0; m < C::kNM; ++m) {
        const int i = i0 + (m0 + m) * 16 + r;
#pragma unroll
        for (int n = 0; n < C::kNN; ++n) {
            const int j = j0 + (n0 + n) * 16 + 4 * c4;
            uint2 o;
            o.x = bf16_pack2(acc[m][n][0], acc[m][n][1]);
            o.y = bf16_pack2(acc[m][n][2], acc[m][n][3]);
            if (i < I) *reinterpret_cast<uint2*>(out + (size_t)i * J + j) = o;
        }
    }
}

// ----------------------------------------------------------------- launch --

template <typename K>
static hipError_t allow_lds(K kernel, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// big tile: 256x256, 8 waves of 128x64;  small tile: 128x128, 4 waves of 64x64
#define JET_BIG 2, 4, 8, 4
#define JET_SMALL 2, 2, 4, 4
#define JET_SMALL_DEEP 2, 2, 4, 4, 4   /* four stages, one workgroup per CU: copies three steps ahead */
#define JET_HALF 4, 1, 2, 4, 4         /* 128x64 tile, 4 waves of 32x64, four stages (six measured the same) */
#define JET_STRIP_SMALL 2, 2, 4, 4   /* 32-row blocks, two workgroups per CU */
#define JET_STRIP_WIDE 4, 2, 7, 5    /* 64-row blocks */
using StripSmall = StripCfg<JET_STRIP_SMALL>;
using StripWide = StripCfg<JET_STRIP_WIDE>;
using BigCfg = TileCfg<JET_BIG>;
using SmallCfg = TileCfg<JET_SMALL>;
using SmallDeepCfg = TileCfg<JET_SMALL_DEEP>;
using HalfCfg = TileCfg<JET_HALF>;

// compute units of the current device (256 on MI355X), asked once per process
static int compute_units() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
            v = 256;
        return v;
    }();
    return n;
}

// out has row pitch ldo (>= J): the launches below also run on row or column ranges of a larger problem
template <int SB_MODE>
static hipError_t launch_tile(const uint8_t* A, const float* sa, const uint8_t* B, const float* sb,
                              uint16_t* o, long I, long J, long R, long ldo, hipStream_t st) {
    // shape-only choice: the big tile when it divides J and fills the 256 CUs.  The grid
    // is persistent: at most one resident set of workgroups, each walking its tile list.
    const int cus = compute_units();
    const long G = R / kGroup;
    const long big_tiles = ((I + 255) / 256) * (J / 256);
    if (J % 256 == 0 && big_tiles >= 224) {
        const int ti = (int)((I + 255) / 256), tj = (int)(J / 256);
        // A last round that fills at most half of the CUs (896 tiles = 3.5 rounds for the 14336-wide
        // WGrads) would cost a whole round: split those tiles off as whole tile rows or tile columns
        // and run them as 128x128 tiles, two workgroups per CU.  An output element takes the same
        // chain in either kernel.
        const long tail = big_tiles % cus;
        if (big_tiles > cus && tail > 0 && tail <= cus / 2) {
            if (tail % tj == 0) {
                const long i_main = (ti - tail / tj) * 256;
                hipError_t e = launch_tile<SB_MODE>(A, sa, B, sb, o, i_main, J, R, ldo, st);
                if (e != hipSuccess) return e;
                return launch_tile<SB_MODE>(A + i_main * R, sa + i_main * G, B, sb, o + i_main * ldo, I - i_main, J,
                                            R, ldo, st);
            }
            if (tail % ti == 0) {
                const long j_main = (tj - tail / ti) * 256;
                hipError_t e = launch_tile<SB_MODE>(A, sa, B, sb, o, I, j_main, R, ldo, st);
                if (e != hipSuccess) return e;
                const float* sb_tail = sb + (SB_MODE == kSbBlock ? (j_main / kGroup) * G : j_main * G);
                return launch_tile<SB_MODE>(A, sa, B + j_main * R, sb_tail, o + j_main, I, J - j_main, R, ldo, st);
            }
        }
        const long wgs = std::min<long>((long)ti * tj, (long)cus * BigCfg::kOccupancy);
        hipLaunchKernelGGL((gemm_tile_kernel<SB_MODE, JET_BIG>), dim3((unsigned)wgs),
                           dim3(BigCfg::kThreads), BigCfg::kLdsBytes, st, A, sa, B, sb, o, (int)I, (int)ldo,
                           (int)R, ti, tj);
    } else {
        const int ti = (int)((I + 127) / 128), tj = (int)(J / 128);
        if (SB_MODE == kSbBlock && (long)ti * tj <= cus / 2) {
            // 128x128 tiles would leave half of the CUs idle: 128x64 tiles, one per CU
            hipLaunchKernelGGL((gemm_tile_kernel<kSbBlock, JET_HALF>), dim3((unsigned)(ti * tj * 2)),
                               dim3(HalfCfg::kThreads), HalfCfg::kLdsBytes, st, A, sa, B, sb, o, (int)I, (int)ldo,
                               (int)R, ti, tj * 2);
            return hipGetLastError();
        }
        if ((long)ti * tj <= cus) {
            // at most one workgroup per CU anyway: spend the LDS on two more stages, so that operands
            // that come from HBM (decode batches against cold weights) are fetched three steps ahead
            hipLaunchKernelGGL((gemm_tile_kernel<SB_MODE, JET_SMALL_DEEP>), dim3((unsigned)(ti * tj)),
                               dim3(SmallDeepCfg::kThreads), SmallDeepCfg::kLdsBytes, st, A, sa, B, sb, o, (int)I,
                               (int)ldo, (int)R, ti, tj);
            return hipGetLastError();
        }
        const long wgs = std::min<long>((long)ti * tj, (long)cus * SmallCfg::kOccupancy);
        hipLaunchKernelGGL((gemm_tile_kernel<SB_MODE, JET_SMALL>), dim3((unsigned)wgs),
                           dim3(SmallCfg::kThreads), SmallCfg::kLdsBytes, st, A, sa, B, sb, o, (int)I,
                           (int)ldo, (int)R, ti, tj);
    }
    return hipGetLastError();
}

hipError_t launch_gemm(const uint8_t* A, const float* sa, const uint8_t* B, const float* sb,
                       int sb_mode, void* out, long I, long J, long R, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        hipError_t e = allow_lds(gemm_tile_kernel<kSbBlock, JET_BIG>, BigCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbRow, JET_BIG>, BigCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbBlock, JET_SMALL>, SmallCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbRow, JET_SMALL>, SmallCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbBlock, JET_SMALL_DEEP>, SmallDeepCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbRow, JET_SMALL_DEEP>, SmallDeepCfg::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_tile_kernel<kSbBlock, JET_HALF>, HalfCfg::kLdsBytes);
#define JET_SK_ATTR(D, W, RMT, AB) \
    if (e == hipSuccess) e = allow_lds(gemm_skinny_kernel<D, W, RMT, AB>, sk_lds_bytes(D, W, RMT))
        JET_SK_ATTR(6, 4, 1, 1); JET_SK_ATTR(6, 4, 1, 2);
        JET_SK_ATTR(3, 8, 1, 1); JET_SK_ATTR(3, 8, 1, 2);
        JET_SK_ATTR(1, 8, 1, 1); JET_SK_ATTR(1, 8, 1, 2);
        JET_SK_ATTR(2, 8, 2, 3); JET_SK_ATTR(2, 8, 2, 4);
#undef JET_SK_ATTR
        if (e == hipSuccess) e = allow_lds(gemm_strip_kernel<JET_STRIP_SMALL>, StripSmall::kLdsBytes);
        if (e == hipSuccess) e = allow_lds(gemm_strip_kernel<JET_STRIP_WIDE>, StripWide::kLdsBytes);
        attr_err = e;
    });
    if (attr_err != hipSuccess) return attr_err;

    uint16_t* o = static_cast<uint16_t*>(out);
    // decode: a workgroup per 16-column strip; shape-only choice of ring depth / wave count
    // (17-32 rows with more strips than CUs go to the strip kernel below: measured faster)
    if ((I <= 16 || (I <= 32 && J / 16 <= 256)) && sb_mode == kSbBlock) {
        const unsigned strips = (unsigned)(J / 16);
#define JET_SKINNY_AB(D, W, RMT, AB)                                                                          \
    hipLaunchKernelGGL((gemm_skinny_kernel<D, W, RMT, AB>), dim3(strips), dim3(64 * W), sk_lds_bytes(D, W, RMT), \
                       st, A, sa, B, sb, o, (int)I, (int)J, (int)R)
        // copy only the 8-row activation blocks that hold a row of the batch
#define JET_SKINNY(D, W, RMT)                                        \
    do {                                                             \
        if ((I + 7) / 8 < 2 * RMT) JET_SKINNY_AB(D, W, RMT, 2 * RMT - 1); \
        else JET_SKINNY_AB(D, W, RMT, 2 * RMT);                      \
    } while (0)
        if (I > 16) {
            JET_SKINNY(2, 8, 2);
        } else if (strips > 256) {
            JET_SKINNY(1, 8, 1);                        // two workgroups (16 waves) per CU
        } else if (R >= 1024) {
            JET_SKINNY(3, 8, 1);
        } else {
            JET_SKINNY(6, 4, 1);
        }
#undef JET_SKINNY
#undef JET_SKINNY_AB
        return hipGetLastError();
    }
    // batches of 65-256 rows against a wide weight matrix (a hundred 128x128 tiles or more) are
    // faster on the tile kernel (measured, gate/up 14336x4096: 30 against 45 us at 128 rows, 30
    // against 74 us at 256 rows); narrower ones (4096 columns) stay on the strip kernel
    const bool wide_batch = I > 64 && ((I + 127) / 128) * (J / 128) >= 100;
    if (I <= 256 && sb_mode == kSbBlock && !wide_batch) {
        // decode batches: 32- or 64-row blocks x 32-column strips
        // 32-row blocks for up to 32 rows, and for larger batches whose 64-row grid would leave
        // half of the CUs without a workgroup (shape-only rule; measured at 64 rows, N = 4096: 9.7
        // against 12.8 us)
        const long wide_wgs = ((I + StripWide::BM - 1) / StripWide::BM) * (J / 32);
        if (I <= 32 || wide_wgs <= 128) {
            const int rbs = (int)((I + StripSmall::BM - 1) / StripSmall::BM);
            hipLaunchKernelGGL((gemm_strip_kernel<JET_STRIP_SMALL>), dim3((unsigned)(rbs * (J / 32))), dim3(512),
                               StripSmall::kLdsBytes, st, A, sa, B, sb, o, (int)I, (int)J, (int)R, rbs);
        } else {
            const int rbs = (int)((I + StripWide::BM - 1) / StripWide::BM);
            hipLaunchKernelGGL((gemm_strip_kernel<JET_STRIP_WIDE>), dim3((unsigned)(rbs * (J / 32))), dim3(512),
                               StripWide::kLdsBytes, st, A, sa, B, sb, o, (int)I, (int)J, (int)R, rbs);
        }
        return hipGetLastError();
    }
    if (sb_mode == kSbBlock) return launch_tile<kSbBlock>(A, sa, B, sb, o, I, J, R, J, st);
    return launch_tile<kSbRow>(A, sa, B, sb, o, I, J, R, J, st);
}

}  // namespace jet
