// Device-side helpers: vector loads/stores of fp32 / bf16 runs, the update formula, and the
// ballot-based packing of per-lane sign bits into the 64-coordinates-per-word message format.
#pragma once
#include "common.h"

namespace ssv {

// ---- streaming accesses --------------------------------------------------------------------
// Every gradient, momentum and weight element is touched once per step, so the 8- and 16-byte
// accesses carry the non-temporal hint: measured on MI355X this is worth about 10% of HBM
// bandwidth on the fused step (the lines do not linger in L2 / Infinity Cache).
template <typename V>
__device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V>
__device__ __forceinline__ void stream_store(V* p, V v) { __builtin_nontemporal_store(v, p); }

// Wait until every memory operation this wave has issued has completed.  Placed after each row
// load of the fused step it keeps ONE load per wave in flight: with 16-20 waves per CU that is
// already enough bytes in flight to cover HBM latency, and on MI355X the fused step then runs
// about 10% faster than with 16 loads per wave queued up (deep per-wave queues lower the
// sustained HBM rate of this 30-stream read/write mix; measured, see the design notes).
__device__ __forceinline__ void drain_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- loads: VEC consecutive elements starting at p, widened to fp32 ------------------------
// Vector forms need p aligned to min(16, VEC * sizeof(element)) bytes.
template <int VEC>
__device__ __forceinline__ void load_vals(const float* __restrict__ p, float (&o)[VEC]) {
    if constexpr (VEC == 1) {
        o[0] = p[0];
    } else {
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            f32x4 t = stream_load(reinterpret_cast<const f32x4*>(p + 4 * q));
            o[4 * q + 0] = t.x; o[4 * q + 1] = t.y; o[4 * q + 2] = t.z; o[4 * q + 3] = t.w;
        }
    }
}

template <int VEC>
__device__ __forceinline__ void load_vals(const bf16* __restrict__ p, float (&o)[VEC]) {
    if constexpr (VEC == 1) {
        o[0] = bf16_bits_to_f32(p[0].bits);
    } else if constexpr (VEC == 4) {
        u32x2 t = stream_load(reinterpret_cast<const u32x2*>(p));
        o[0] = __uint_as_float(t.x << 16); o[1] = __uint_as_float(t.x & 0xffff0000u);
        o[2] = __uint_as_float(t.y << 16); o[3] = __uint_as_float(t.y & 0xffff0000u);
    } else {
        static_assert(VEC == 8, "bf16 runs are 1, 4 or 8 long");
        u32x4 t = stream_load(reinterpret_cast<const u32x4*>(p));
        o[0] = __uint_as_float(t.x << 16); o[1] = __uint_as_float(t.x & 0xffff0000u);
        o[2] = __uint_as_float(t.y << 16); o[3] = __uint_as_float(t.y & 0xffff0000u);
        o[4] = __uint_as_float(t.z << 16); o[5] = __uint_as_float(t.z & 0xffff0000u);
        o[6] = __uint_as_float(t.w << 16); o[7] = __uint_as_float(t.w & 0xffff0000u);
    }
}

// Tail form: only the first n (< VEC allowed) elements exist; the rest read as 0.
template <typename T, int VEC>
__device__ __forceinline__ void load_vals_guarded(const T* __restrict__ p, int n, float (&o)[VEC]) {
    if (n >= VEC) {
        load_vals<VEC>(p, o);
    } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float one[1] = {0.0f};
            if (c < n) load_vals<1>(p + c, one);
            o[c] = one[0];
        }
    }
}

// ---- stores --------------------------------------------------------------------------------
template <int VEC>
__device__ __forceinline__ void store_vals(float* __restrict__ p, const float (&o)[VEC]) {
    if constexpr (VEC == 1) {
        p[0] = o[0];
    } else {
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            f32x4 t = {o[4 * q + 0], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]};
            stream_store(reinterpret_cast<f32x4*>(p + 4 * q), t);
        }
    }
}

template <int VEC>
__device__ __forceinline__ void store_vals(bf16* __restrict__ p, const float (&o)[VEC]) {
    if constexpr (VEC == 1) {
        p[0].bits = (uint16_t)f32_to_bf16_bits(o[0]);
    } else if constexpr (VEC == 4) {
        u32x2 t = {f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16),
                   f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16)};
        stream_store(reinterpret_cast<u32x2*>(p), t);
    } else {
        static_assert(VEC == 8, "bf16 runs are 1, 4 or 8 long");
        u32x4 t = {f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16),
                   f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16),
                   f32_to_bf16_bits(o[4]) | (f32_to_bf16_bits(o[5]) << 16),
                   f32_to_bf16_bits(o[6]) | (f32_to_bf16_bits(o[7]) << 16)};
        stream_store(reinterpret_cast<u32x4*>(p), t);
    }
}

template <typename T, int VEC>
__device__ __forceinline__ void store_vals_guarded(T* __restrict__ p, int n, const float (&o)[VEC]) {
    if (n >= VEC) {
        store_vals<VEC>(p, o);
    } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            if (c < n) {
                float one[1] = {o[c]};
                store_vals<1>(p + c, one);
            }
        }
    }
}

// ---- x <- x - lr (s + wd x), s = +1 if plus else -1 (Algorithm 1, "update parameters") ------
__device__ __forceinline__ float sign_update(float x, bool plus, float lr, float wd) {
    if (wd == 0.0f) return x + (plus ? -lr : lr);
    float t = fmaf(wd, x, plus ? 1.0f : -1.0f);
    return fmaf(-lr, t, x);
}

// ---- packing -------------------------------------------------------------------------------
// spread<VEC>(x): move bit i of x (i < 64 / VEC) to bit VEC * i.
template <int VEC>
__device__ __forceinline__ uint64_t spread_bits(uint64_t x) {
    if constexpr (VEC == 1) {
        return x;
    } else if constexpr (VEC == 4) {
        x = (x | (x << 24)) & 0x000000FF000000FFull;
        x = (x | (x << 12)) & 0x000F000F000F000Full;
        x = (x | (x << 6)) & 0x0303030303030303ull;
        x = (x | (x << 3)) & 0x1111111111111111ull;
        return x;
    } else {
        static_assert(VEC == 8, "1, 4 or 8 coordinates per lane");
        x = (x | (x << 28)) & 0x0000000F0000000Full;
        x = (x | (x << 14)) & 0x0003000300030003ull;
        x = (x | (x << 7)) & 0x0101010101010101ull;
        return x;
    }
}

// A wavefront owns 64 * VEC consecutive coordinates, lane l owning VEC * l .. VEC * l + VEC - 1
// with bit b[c] for its c-th one.  Returns in words[k] the k-th 64-bit word of that run (bit i of
// word k <-> coordinate 64 k + i).  One wave ballot per c; the interleave is scalar work.
template <int VEC>
__device__ __forceinline__ void pack_tile(const uint32_t (&b)[VEC], uint64_t (&words)[VEC]) {
    uint64_t ballots[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) ballots[c] = __ballot(b[c] != 0);
    constexpr int kLanesPerWord = kWave / VEC;
    constexpr uint64_t kChunkMask = (VEC == 1) ? ~0ull : ((1ull << (kLanesPerWord % 64)) - 1ull);
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        uint64_t w = 0;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            uint64_t chunk = (VEC == 1) ? ballots[c] : ((ballots[c] >> (k * kLanesPerWord)) & kChunkMask);
            w |= spread_bits<VEC>(chunk) << c;
        }
        words[k] = w;
    }
}

// Lane k (< VEC) stores word k of the tile if it lies inside the row of W words.
template <int VEC>
__device__ __forceinline__ void store_tile_words(uint64_t* __restrict__ row, int64_t tile, int64_t W,
                                                 int lane, const uint64_t (&words)[VEC]) {
    uint64_t mine = words[0];
#pragma unroll
    for (int k = 1; k < VEC; ++k) mine = (lane == k) ? words[k] : mine;
    int64_t w = tile * VEC + lane;
    if (lane < VEC && w < W) row[w] = mine;
}

// Physical block id -> logical block id.  Workgroups are handed to the 8 XCDs round-robin; with
// the remap on, XCD k walks the k-th contiguous eighth of the logical blocks, so neighbouring
// tiles (which share cache lines when rows are not line-aligned) meet in one XCD's L2.
__device__ __forceinline__ int64_t logical_block(int64_t phys, int64_t nblocks_logical, int remap) {
    if (!remap) return phys;
    int64_t chunk = (nblocks_logical + 7) / 8;
    return (phys % 8) * chunk + phys / 8;
}

}  // namespace ssv
