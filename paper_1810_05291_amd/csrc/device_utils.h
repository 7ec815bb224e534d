// Device-side helpers: vector loads/stores of fp32 / bf16 runs, the update formula, and the
// packing of per-lane sign bits into the 64-coordinates-per-word message format.
#pragma once
#include "common.h"

namespace ssv {

// ---- streaming accesses --------------------------------------------------------------------
// Every gradient, momentum and weight element is touched once per step, so the 8- and 16-byte
// accesses carry the non-temporal hint: measured on MI355X this is worth about 10% of HBM
// bandwidth on the fused step (the lines do not linger in L2 / Infinity Cache).
// Every pointer that reaches these helpers is device (global) memory.  Saying so in the type -- instead of leaving
// a generic pointer, which is all the compiler knows about a pointer it loaded from a table -- gives global_load /
// global_store with "scalar base + 32-bit lane offset" addressing rather than flat instructions on 64-bit
// per-lane addresses (which also cost two registers per live pointer).
#define SSV_GLOBAL __attribute__((address_space(1)))
#define SSV_CONSTANT __attribute__((address_space(4)))
template <typename V>
__device__ __forceinline__ V stream_load(const V* p) {
    return __builtin_nontemporal_load((const SSV_GLOBAL V*)p);
}
template <typename V>
__device__ __forceinline__ void stream_store(V* p, V v) {
    __builtin_nontemporal_store(v, (SSV_GLOBAL V*)p);
}
// A 64-bit value (a device address) from a read-only table at a wave-uniform index: a scalar load.
__device__ __forceinline__ uint64_t uniform_table_entry(const void* table, int64_t index) {
    return ((const SSV_CONSTANT uint64_t*)table)[index];
}

// Wait until every memory operation this wave has issued has completed.  Placed after each row
// load of the fused step it keeps ONE load per wave in flight: with 16-20 waves per CU that is
// already enough bytes in flight to cover HBM latency, and on MI355X the fused step then runs
// about 10% faster than with 16 loads per wave queued up (deep per-wave queues lower the
// sustained HBM rate of this 30-stream read/write mix: 5.3 vs 5.8-6.0 TB/s measured).
__device__ __forceinline__ void drain_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- loads: VEC consecutive elements starting at p, widened to fp32 ------------------------
// Vector forms need p aligned to min(16, VEC * sizeof(element)) bytes.
template <int VEC>
__device__ __forceinline__ void load_vals(const float* __restrict__ p, float (&o)[VEC]) {
    if constexpr (VEC == 1) {
        o[0] = *(const SSV_GLOBAL float*)p;
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
        o[0] = bf16_bits_to_f32(((const SSV_GLOBAL bf16*)p)->bits);
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
        *(SSV_GLOBAL float*)p = o[0];
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
        ((SSV_GLOBAL bf16*)p)->bits = (uint16_t)f32_to_bf16_bits(o[0]);
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

// ---- x <- x - lr (s + wd x), s = +1 if plus else -1 (Algorithm 1, the update line) ------
__device__ __forceinline__ float sign_update(float x, bool plus, float lr, float wd) {
    if (wd == 0.0f) return x + (plus ? -lr : lr);
    float t = fmaf(wd, x, plus ? 1.0f : -1.0f);
    return fmaf(-lr, t, x);
}

// ---- packing -------------------------------------------------------------------------------
// A wavefront owns a tile of 64 * VEC consecutive coordinates, lane l owning VEC * l .. VEC * l +
// VEC - 1 with bit b[c] for its c-th one.  The tile's words (bit i of word k <-> coordinate
// 64 k + i of the tile) are written to row[tile * VEC + k], for the words that lie inside the
// row of W words.
//
// VEC = 1: the wave ballot IS the word.
// VEC = 4: each lane shifts its 4-bit group to its place inside the dword that 8 neighbouring
// lanes share, and three DPP steps (lane ^ 1, lane ^ 2, mirror inside the half row) OR the eight
// groups together; the first lane of every eight then stores its dword.  A handful of vector
// instructions per tile; an interleave of four ballot masks on the scalar unit costs ~200.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_or(uint32_t v) {
    return v | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// Plain stores on purpose: with the non-temporal hint these 32-byte pieces reach memory as partial-line writes (the
// sign-only form then writes 1.21 x its packed bytes) and the momentum and bit-plane kernels run 0.5-2% slower.
template <int VEC>
__device__ __forceinline__ void pack_store_tile(uint64_t* __restrict__ row, int64_t tile, int64_t W, int lane,
                                                const uint32_t (&b)[VEC]) {
    if constexpr (VEC == 1) {
        const uint64_t word = __ballot(b[0] != 0);
        if (lane == 0 && tile < W) row[tile] = word;
    } else {
        static_assert(VEC == 4, "1 or 4 coordinates per lane");
        uint32_t v = (b[0] | (b[1] << 1) | (b[2] << 2) | (b[3] << 3)) << (4 * (lane & 7));
        v = dpp_or<0xB1>(v);     // quad_perm [1,0,3,2]
        v = dpp_or<0x4E>(v);     // quad_perm [2,3,0,1]
        v = dpp_or<0x141>(v);    // row_half_mirror
        const int64_t dw = tile * 8 + (lane >> 3);          // dword index inside the packed row
        if ((lane & 7) == 0 && (dw >> 1) < W) reinterpret_cast<uint32_t*>(row)[dw] = v;
    }
}

}  // namespace ssv
