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
#include "device_utils.h"

namespace ssv {

// Packed rows are read once: streaming loads.  Unlike the fused gradient step, this pure-read
// stream runs fastest with all eight row loads of a batch in flight.
template <typename V>
__device__ __forceinline__ V row_load(const V* p) { return stream_load(p); }

template <int PW>
__device__ __forceinline__ void load_slices(const uint32_t* __restrict__ p, int nv, uint32_t (&r)[PW]) {
    // nv = number of this lane's dwords that exist in the row (0, 2 or 4; whole 64-bit words)
    if constexpr (PW == 2) {
        if (nv > 0) {
            u32x2 t = row_load(reinterpret_cast<const u32x2*>(p));
            r[0] = t.x; r[1] = t.y;
        } else {
            r[0] = 0; r[1] = 0;
        }
    } else {
        static_assert(PW == 4, "8- or 16-byte pieces");
        if (nv == 4) {
            u32x4 t = row_load(reinterpret_cast<const u32x4*>(p));
            r[0] = t.x; r[1] = t.y; r[2] = t.z; r[3] = t.w;
        } else if (nv == 2) {
            u32x2 t = row_load(reinterpret_cast<const u32x2*>(p));
            r[0] = t.x; r[1] = t.y; r[2] = 0; r[3] = 0;
        } else {
            r[0] = 0; r[1] = 0; r[2] = 0; r[3] = 0;
        }
    }
}

// full adder on bit planes: s <- a ^ b ^ c, returns majority(a, b, c)
__device__ __forceinline__ uint32_t csa(uint32_t& s, uint32_t a, uint32_t b, uint32_t c) {
    uint32_t carry = (a & b) | (c & (a ^ b));
    s = a ^ b ^ c;
    return carry;
}

template <int PW, int NPL>
__device__ __forceinline__ void add_eight_rows(uint32_t (&pl)[NPL][PW], const uint32_t (&r)[8][PW]) {
#pragma unroll
    for (int q = 0; q < PW; ++q) {
        uint32_t ones = pl[0][q], twos = pl[1][q], fours = pl[2][q];
        uint32_t c1 = csa(ones, ones, r[0][q], r[1][q]);
        uint32_t c2 = csa(ones, ones, r[2][q], r[3][q]);
        uint32_t c3 = csa(ones, ones, r[4][q], r[5][q]);
        uint32_t c4 = csa(ones, ones, r[6][q], r[7][q]);
        uint32_t d1 = csa(twos, twos, c1, c2);
        uint32_t d2 = csa(twos, twos, c3, c4);
        uint32_t e = csa(fours, fours, d1, d2);
        pl[0][q] = ones; pl[1][q] = twos; pl[2][q] = fours;
#pragma unroll
        for (int p = 3; p < NPL - 1; ++p) {
            uint32_t t = pl[p][q] & e;
            pl[p][q] ^= e;
            e = t;
        }
        pl[NPL - 1][q] ^= e;   // the preload bound guarantees no carry leaves the top plane
    }
}

template <typename XT, int XV>
__device__ __forceinline__ void apply_piece(XT* __restrict__ xp, int n, uint32_t bits, float lr, float wd) {
    float xv[XV];
    load_vals_guarded<XT, XV>(xp, n, xv);
#pragma unroll
    for (int c = 0; c < XV; ++c) xv[c] = sign_update(xv[c], ((bits >> c) & 1u) != 0, lr, wd);
    store_vals_guarded<XT, XV>(xp, n, xv);
}

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
        uint32_t* o = reinterpret_cast<uint32_t*>(a.vote_out) + dw0;
        if constexpr (PW == 4) {
            if (FULL || nv == 4) {
                u32x4 w = {vt[0], vt[1], vt[2], vt[3]};
                *reinterpret_cast<u32x4*>(o) = w;
            } else {
                u32x2 w = {vt[0], vt[1]};
                *reinterpret_cast<u32x2*>(o) = w;
            }
        } else {
            u32x2 w = {vt[0], vt[1]};
            *reinterpret_cast<u32x2*>(o) = w;
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

// One access of the weight walk of a wave tile: lane l owns the XV weights at coordinate offset
// (i * 64 + l) * XV of the tile; their vote bits sit in dword off / 32 of the tile, which lane off / 32
// holds in `vt`.  Every lane of the wave must be active here (cross-lane read).
template <int XV>
__device__ __forceinline__ uint32_t vote_bits_for(uint32_t vt, int off) {
    const uint32_t w = (uint32_t)__builtin_amdgcn_ds_bpermute((off >> 5) << 2, (int)vt);
    return w >> (off & 31);
}

// Weight walk of a tile that holds the ragged end of the vector: per-element bounds checks.
template <typename XT, int XV>
__device__ __forceinline__ void apply_ragged_tile(XT* __restrict__ xt, int64_t left, uint32_t vt, int lane, float lr,
                                                  float wd) {
    constexpr int kAcc = 32 / XV;                              // accesses that cover the 2048 coordinates
#pragma unroll 4
    for (int i = 0; i < kAcc; ++i) {
        const int off = (i * kWave + lane) * XV;
        const uint32_t bits = vote_bits_for<XV>(vt, off);      // before any per-lane branch
        const int64_t r = left - off;
        const int n = r >= XV ? XV : (r > 0 ? (int)r : 0);
        if (n > 0) {
            float xv[XV];
            load_vals_guarded<XT, XV>(xt + off, n, xv);
#pragma unroll
            for (int c = 0; c < XV; ++c) xv[c] = sign_update(xv[c], ((bits >> c) & 1u) != 0, lr, wd);
            store_vals_guarded<XT, XV>(xt + off, n, xv);
        }
    }
}

// Fused vote + update.  One wavefront per tile of 2048 coordinates (64 dwords of every row); the
// workgroup size (64 or 256 threads) only groups neighbouring tiles on one CU.
// XV = weights per lane per access (4 fp32 / 8 bf16; 1 = any alignment).
// A full tile issues the first half of its weight loads before the row loads, so that they share one
// memory round trip, and the second half behind the vote arithmetic (measured 1-2% faster than loading
// the weights after the vote, and than loading all of them first).
template <int NPL, typename XT, int XV>
__global__ __launch_bounds__(kBlock) void vote_apply_kernel(VoteArgs a) {
    constexpr int kTileCoords = kWave * 32;
    constexpr int kAcc = 32 / XV;                      // weight accesses per lane that cover the tile
    constexpr int kEarly = kAcc / 2;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tile >= a.ntiles) return;                      // wave-uniform
    const int64_t ndw = 2 * a.W;
    const int64_t row_dw = 2 * a.stride_words;
    const int64_t dw = tile * kWave + lane;
    const bool have = dw < ndw;
    const uint32_t* __restrict__ p = reinterpret_cast<const uint32_t*>(a.signs) + dw;
    XT* __restrict__ xt = static_cast<XT*>(a.x) + tile * (int64_t)kTileCoords;
    const int64_t left = a.d - tile * (int64_t)kTileCoords;      // > 0: the tile exists
    const bool full = left >= kTileCoords;                        // wave-uniform

    float xv[kAcc][XV];
    if (full) {
#pragma unroll
        for (int i = 0; i < kEarly; ++i) load_vals<XV>(xt + (i * kWave + lane) * XV, xv[i]);
    }

    uint32_t pl[NPL][1];
#pragma unroll
    for (int pnum = 0; pnum < NPL; ++pnum) pl[pnum][0] = ((a.init >> pnum) & 1u) ? 0xffffffffu : 0u;
    for (int r0 = 0; r0 < a.M; r0 += 8) {
        uint32_t cur[8][1];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            cur[i][0] = (have && r0 + i < a.M) ? row_load(p + (int64_t)(r0 + i) * row_dw) : 0u;
        add_eight_rows<1, NPL>(pl, cur);
    }
    const int64_t rem = a.d - dw * 32;
    const uint32_t mask = rem >= 32 ? 0xffffffffu : (rem > 0 ? ((1u << (int)rem) - 1u) : 0u);
    const uint32_t vt = pl[NPL - 1][0] & mask;
    if (a.vote_out != nullptr && have) reinterpret_cast<uint32_t*>(a.vote_out)[dw] = vt;

    // all 64 lanes are active again here: the cross-lane reads below need every lane
    if (full) {
#pragma unroll
        for (int i = kEarly; i < kAcc; ++i) load_vals<XV>(xt + (i * kWave + lane) * XV, xv[i]);
#pragma unroll
        for (int i = 0; i < kAcc; ++i) {
            const int off = (i * kWave + lane) * XV;
            const uint32_t bits = vote_bits_for<XV>(vt, off);
#pragma unroll
            for (int c = 0; c < XV; ++c) xv[i][c] = sign_update(xv[i][c], ((bits >> c) & 1u) != 0, a.lr, a.wd);
            store_vals<XV>(xt + off, xv[i]);
        }
    } else {
        apply_ragged_tile<XT, XV>(xt, left, vt, lane, a.lr, a.wd);
    }
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
