// Device code shared by the kernels that vote on packed sign rows (vote_kernels.hip, multi_kernels.hip): the
// carry-save adder network on bit planes and the vote + update of one wave tile.
#pragma once
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

// Vote + update of one wave tile: 64 consecutive dwords of every packed row (2048 coordinates), one dword per lane.
//   p       this lane's dword of row 0 (rows are row_dw dwords apart);  have = the dword exists in the rows
//   rem     coordinates of the vector from this lane's first bit on (<= 0: none); masks the padding bits
//   xt      weight of the tile's first coordinate;  left = coordinates from there to the end of the vector (> 0)
//   vote_dw where this lane's vote dword goes, or nullptr
// XV = weights per lane per access (4 fp32 / 8 bf16; 1 = any alignment).  Every lane of the wave must call this.
// A full tile issues the first half of its weight loads before the row loads, so that they share one memory round
// trip, and the second half behind the vote arithmetic (measured 1-2% faster than loading the weights after the
// vote, and than loading all of them first).
template <int NPL, typename XT, int XV>
__device__ __forceinline__ void vote_apply_tile(const uint32_t* __restrict__ p, int64_t row_dw, int M, uint32_t init,
                                                bool have, int64_t rem, XT* __restrict__ xt, int64_t left,
                                                uint32_t* vote_dw, float lr, float wd, int lane) {
    constexpr int kTileCoords = kWave * 32;
    constexpr int kAcc = 32 / XV;                      // weight accesses per lane that cover the tile
    constexpr int kEarly = kAcc / 2;
    const bool full = left >= kTileCoords;             // wave-uniform

    float xv[kAcc][XV];
    if (full) {
#pragma unroll
        for (int i = 0; i < kEarly; ++i) load_vals<XV>(xt + (i * kWave + lane) * XV, xv[i]);
    }

    uint32_t pl[NPL][1];
#pragma unroll
    for (int pnum = 0; pnum < NPL; ++pnum) pl[pnum][0] = ((init >> pnum) & 1u) ? 0xffffffffu : 0u;
    for (int r0 = 0; r0 < M; r0 += 8) {
        uint32_t cur[8][1];
#pragma unroll
        for (int i = 0; i < 8; ++i) cur[i][0] = (have && r0 + i < M) ? row_load(p + (int64_t)(r0 + i) * row_dw) : 0u;
        add_eight_rows<1, NPL>(pl, cur);
    }
    const uint32_t mask = rem >= 32 ? 0xffffffffu : (rem > 0 ? ((1u << (int)rem) - 1u) : 0u);
    const uint32_t vt = pl[NPL - 1][0] & mask;
    if (vote_dw != nullptr && have) *vote_dw = vt;

    // all 64 lanes are active again here: the cross-lane reads below need every lane
    if (full) {
#pragma unroll
        for (int i = kEarly; i < kAcc; ++i) load_vals<XV>(xt + (i * kWave + lane) * XV, xv[i]);
#pragma unroll
        for (int i = 0; i < kAcc; ++i) {
            const int off = (i * kWave + lane) * XV;
            const uint32_t bits = vote_bits_for<XV>(vt, off);
#pragma unroll
            for (int c = 0; c < XV; ++c) xv[i][c] = sign_update(xv[i][c], ((bits >> c) & 1u) != 0, lr, wd);
            store_vals<XV>(xt + off, xv[i]);
        }
    } else {
        apply_ragged_tile<XT, XV>(xt, left, vt, lane, lr, wd);
    }
}

}  // namespace ssv
