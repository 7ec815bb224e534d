// Server-side kernels on packed sign rows: the majority vote (Algorithm 1, the server's sum and
// sign-of-sum lines), optionally fused with the parameter update, and the
// stand-alone update from a packed vote.
//
// The vote never expands to per-coordinate integers.  A lane holds PW 32-bit slices of the row
// (PW*32 coordinates) and streams the M rows through a carry-save adder network on bit planes:
// plane p holds bit p of the running count of every coordinate.  Eight rows at a time are reduced
// with seven full adders (sum = a^b^c, carry = majority(a,b,c): one three-input bit operation
// each on gfx950) into planes 0..2 and a weight-8 carry that ripples into the upper planes.
// The counter is preloaded with 2^k - T (T = (M+1)/2 the vote threshold, 2^k > M/2), so the top
// plane k is directly [count >= T]: no comparator.
//
// Vote only (vote_kernel): a wavefront owns a tile of 64*PW consecutive dwords of every row; lane
// l loads dwords PW*l .. PW*l+PW-1 of the tile as one 8- or 16-byte piece, so a row access of a
// wave is one contiguous 512 B / 1 KiB run.  Traffic is (M+1)/8 bytes per coordinate.
//
// Fused vote + update (vote_apply_kernel): a wavefront owns 64 consecutive dwords of every row
// (2048 coordinates), one dword per lane, and works alone: no LDS allocation, no barrier.  It then
// walks its 2048 weights in contiguous 1 KiB accesses; the lane that updates weights 4 l .. 4 l + 3
// of an access fetches the vote dword that holds their bits from the lane that computed it with one
// cross-lane read.  Traffic is M/8 + 8 bytes per coordinate at fp32 and is dominated by the weights,
// so the narrow 4-byte row loads cost nothing, while the small independent tiles (12,479 waves at the
// resnet50 size instead of 3,120 barrier-synchronised workgroups) keep every CU busy through the
// 40 microseconds the kernel lasts: 77% of the HBM peak against 69% for the workgroup-tile form, and
// wider row loads (8 or 16 bytes per lane, 4096 or 8192 coordinates per wave) measured 3-6 points lower.
#include "vote_tiles.h"

namespace ssv {

// FULL = every lane of the wave has all its PW dwords inside the row (no per-lane bounds checks).
template <int PW, int NPL, bool FULL>
__device__ __forceinline__ void vote_tile(const VoteArgs& a, int64_t dw0, int nv) {
    const int64_t row_dw = 2 * a.stride_words;
    const uint32_t* __restrict__ p = reinterpret_cast<const uint32_t*>(a.signs) + dw0;
    constexpr int kFullNv = PW;

    uint32_t pl[NPL][PW];
#pragma unroll
    for (int pnum = 0; pnum < NPL; ++pnum)
#pragma unroll
        for (int q = 0; q < PW; ++q) pl[pnum][q] = ((a.init >> pnum) & 1u) ? 0xffffffffu : 0u;

    // Batches of eight rows.  The loads of the next batch are written after the adder network of
    // the current one; the compiler is free to issue them early (loads only, nothing aliases).
    uint32_t cur[8][PW];
#pragma unroll
    for (int i = 0; i < 8; ++i) load_slices<PW>(p + (int64_t)i * row_dw, (i < a.M) ? (FULL ? kFullNv : nv) : 0, cur[i]);
    for (int r0 = 0; r0 < a.M; r0 += 8) {
        uint32_t nxt[8][PW];
        const int rn = r0 + 8;
        add_eight_rows<PW, NPL>(pl, cur);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            load_slices<PW>(p + (int64_t)(rn + i) * row_dw, (rn + i < a.M) ? (FULL ? kFullNv : nv) : 0, nxt[i]);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < PW; ++q) cur[i][q] = nxt[i][q];
    }

    if (FULL || nv > 0) {
        uint32_t vt[PW];
#pragma unroll
        for (int q = 0; q < PW; ++q) {
            const int64_t rem = a.d - (dw0 + q) * 32;
            const uint32_t mask = rem >= 32 ? 0xffffffffu : (rem > 0 ? ((1u << (int)rem) - 1u) : 0u);
            vt[q] = pl[NPL - 1][q] & mask;
        }
        // Non-temporal like the loads: with plain stores the vote's output, 0.4% of its traffic, costs the d = 2^30,
        // M = 255 vote 4-5% of its time (5.47-5.63 -> 5.18-5.38 ms); with no stores at all it would take 4.90 ms.
        uint32_t* o = reinterpret_cast<uint32_t*>(a.vote_out) + dw0;
        if constexpr (PW == 4) {
            if (FULL || nv == 4) {
                u32x4 w = {vt[0], vt[1], vt[2], vt[3]};
                stream_store(reinterpret_cast<u32x4*>(o), w);
            } else {
                u32x2 w = {vt[0], vt[1]};
                stream_store(reinterpret_cast<u32x2*>(o), w);
            }
        } else {
            u32x2 w = {vt[0], vt[1]};
            stream_store(reinterpret_cast<u32x2*>(o), w);
        }
    }
}

template <int PW, int NPL>
__global__ __launch_bounds__(kBlock) void vote_kernel(VoteArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t tile = (int64_t)blockIdx.x * (blockDim.x / kWave) + wave;
    if (tile >= a.ntiles) return;
    const int64_t ndw = 2 * a.W;
    const int64_t dw0 = (tile * kWave + lane) * PW;
    if ((tile + 1) * (int64_t)(kWave * PW) <= ndw) {          // wave-uniform: the whole tile is inside the row
        vote_tile<PW, NPL, true>(a, dw0, PW);
    } else {
        const int64_t left = ndw - dw0;
        vote_tile<PW, NPL, false>(a, dw0, left >= PW ? PW : (left > 0 ? (int)left : 0));
    }
}

// Fused vote + update.  One wavefront per tile of 2048 coordinates (64 dwords of every row); the
// workgroup size (64 or 256 threads) only groups neighbouring tiles on one CU.  The tile body is vote_apply_tile.
template <int NPL, typename XT, int XV>
__global__ __launch_bounds__(kBlock) void vote_apply_kernel(VoteArgs a) {
    constexpr int kTileCoords = kWave * 32;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tile >= a.ntiles) return;                      // wave-uniform
    const int64_t dw = tile * kWave + lane;
    const bool have = dw < 2 * a.W;
    uint32_t* vote_dw = a.vote_out != nullptr ? reinterpret_cast<uint32_t*>(a.vote_out) + dw : nullptr;
    vote_apply_tile<NPL, XT, XV>(reinterpret_cast<const uint32_t*>(a.signs) + dw, 2 * a.stride_words, a.M, a.init, have,
                                 a.d - dw * 32, static_cast<XT*>(a.x) + tile * (int64_t)kTileCoords,
                                 a.d - tile * (int64_t)kTileCoords, vote_dw, a.lr, a.wd, lane);
}

// A vote that moves less than 512 MiB is over in tens of microseconds: what counts then is how evenly the work
// spreads over the 256 CUs and how soon every CU has loads in flight, not the width of a lane's access.  Such
// votes run with 8-byte row pieces (twice the wavefronts) in single-wave workgroups.  Measured at the resnet50
// size: M = 15, 17.0 -> 10.3 us; M = 31, 31.2 -> 17.7 us (72% of the HBM peak).  Large votes keep 16-byte pieces
// and four-wave workgroups (d = 2^30, M = 255: 78.8% against 66.4% with 8-byte pieces).
static inline bool small_vote(const VoteArgs& a) { return (int64_t)(a.M + 1) * a.d < (1LL << 32); }

template <int PW, int NPL>
static hipError_t launch_vote_only(VoteArgs a, hipStream_t s) {
    const int64_t ndw = 2 * a.W;
    a.ntiles = (ndw + (int64_t)kWave * PW - 1) / ((int64_t)kWave * PW);
    const int waves = small_vote(a) ? 1 : kWavesPerBlock;
    const int64_t grid = (a.ntiles + waves - 1) / waves;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((vote_kernel<PW, NPL>), dim3((unsigned)grid), dim3(waves * kWave), 0, s, a);
    return hipGetLastError();
}

template <int NPL, typename XT, int XV>
static hipError_t launch_vote_apply_one(VoteArgs a, hipStream_t s) {
    const int64_t ndw = 2 * a.W;
    a.ntiles = (ndw + kWave - 1) / kWave;
    // Rows that start on 128-byte boundaries: single-wave workgroups (the dispatcher balances 2048-coordinate
    // tiles one by one).  Otherwise a row piece shares its first and last cache line with the neighbouring
    // tiles, and four-wave workgroups keep those neighbours on one CU (measured: 77.3 vs 76.5% aligned,
    // 72.1 vs 74.8% at the odd natural stride of the resnet50 size).
    const bool lines = reinterpret_cast<uintptr_t>(a.signs) % 128 == 0 && (a.M == 1 || a.stride_words % 16 == 0);
    const int waves = lines ? 1 : kWavesPerBlock;
    const int64_t grid = (a.ntiles + waves - 1) / waves;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((vote_apply_kernel<NPL, XT, XV>), dim3((unsigned)grid), dim3(waves * kWave), 0, s, a);
    return hipGetLastError();
}

template <int NPL>
static hipError_t launch_vote_npl(const VoteArgs& a, int x_dt, bool rows16, bool x_vector_ok, hipStream_t s) {
    if (a.x == nullptr)
        return (rows16 && !small_vote(a)) ? launch_vote_only<4, NPL>(a, s) : launch_vote_only<2, NPL>(a, s);
    if (x_dt == 0)
        return x_vector_ok ? launch_vote_apply_one<NPL, float, 4>(a, s) : launch_vote_apply_one<NPL, float, 1>(a, s);
    return x_vector_ok ? launch_vote_apply_one<NPL, bf16, 8>(a, s) : launch_vote_apply_one<NPL, bf16, 1>(a, s);
}

hipError_t launch_vote(const VoteArgs& a_in, int x_dt, bool rows16, bool x_vector_ok, hipStream_t s) {
    // planes 0..k with 2^k > M/2 and 2^k >= T; template sizes cover M <= 15, 63, 255, 1023
    VoteArgs a = a_in;
    const int T = (a.M + 1) / 2;
    if (a.M <= 15) { a.init = (1u << 3) - T; return launch_vote_npl<4>(a, x_dt, rows16, x_vector_ok, s); }
    if (a.M <= 63) { a.init = (1u << 5) - T; return launch_vote_npl<6>(a, x_dt, rows16, x_vector_ok, s); }
    if (a.M <= 255) { a.init = (1u << 7) - T; return launch_vote_npl<8>(a, x_dt, rows16, x_vector_ok, s); }
    a.init = (1u << 9) - T;
    return launch_vote_npl<10>(a, x_dt, rows16, x_vector_ok, s);
}

// ---- stand-alone update from a packed vote -------------------------------------------------------
// A lane owns XV consecutive coordinates and reads the byte of the vote that holds their bits.
template <typename XT, int XV>
__global__ __launch_bounds__(kBlock) void apply_kernel(ApplyArgs a) {
    const uint8_t* __restrict__ vb = reinterpret_cast<const uint8_t*>(a.vote);
    const int64_t step = (int64_t)gridDim.x * kBlock * XV;      // one pass unless the grid was capped
    for (int64_t j0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * XV; j0 < a.d; j0 += step) {
        const int64_t left = a.d - j0;
        const int n = left >= XV ? XV : (int)left;
        const uint32_t bits = (uint32_t)vb[j0 >> 3] >> (j0 & 7);
        apply_piece<XT, XV>(static_cast<XT*>(a.x) + j0, n, bits, a.lr, a.wd);
    }
}

template <typename XT, int XV>
static hipError_t launch_apply_one(const ApplyArgs& a, hipStream_t s) {
    int64_t threads = (a.d + XV - 1) / XV;
    int64_t grid = (threads + kBlock - 1) / kBlock;
    // Defensive cap: with d <= 2^40 the grid reaches it only beyond 2^38 (1 per lane) .. 2^41 coordinates, far
    // more than one GPU holds; the kernel's stride loop then covers the rest.  No test reaches that loop.
    if (grid > 0x40000000LL) grid = 0x40000000LL;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((apply_kernel<XT, XV>), dim3((unsigned)grid), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_apply(const ApplyArgs& a, int x_dt, bool x_vector_ok, hipStream_t s) {
    if (x_dt == 0) return x_vector_ok ? launch_apply_one<float, 4>(a, s) : launch_apply_one<float, 1>(a, s);
    return x_vector_ok ? launch_apply_one<bf16, 8>(a, s) : launch_apply_one<bf16, 1>(a, s);
}

}  // namespace ssv
