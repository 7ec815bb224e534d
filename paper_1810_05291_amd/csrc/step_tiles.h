// The tile body of the gradient-side kernels: momentum, sign, count over the workers, vote, update for the
// tiles one wavefront holds.  Shared by the flat-vector kernels (step_kernels.hip) and the multi-tensor
// kernel (multi_kernels.hip).
#pragma once
#include "device_utils.h"


namespace ssv {

// Where worker m's row of gradients / momentum starts.  FlatRows: the [M][row_stride] matrices of the flat
// entry points.  TableRows: a.g / a.v point to M device pointers, one per worker (the multi-tensor entry
// point, where every worker's gradient of a tensor is an allocation of its own).
struct FlatRows {
    template <typename GT>
    static __device__ __forceinline__ const GT* g(const StepArgs& a, int m) {
        return static_cast<const GT*>(a.g) + (int64_t)m * a.g_stride;
    }
    static __device__ __forceinline__ float* v(const StepArgs& a, int m) { return a.v + (int64_t)m * a.v_stride; }
};
struct TableRows {
    template <typename GT>
    static __device__ __forceinline__ const GT* g(const StepArgs& a, int m) {
        return reinterpret_cast<const GT*>(uniform_table_entry(a.g, m));
    }
    static __device__ __forceinline__ float* v(const StepArgs& a, int m) {
        return reinterpret_cast<float*>(uniform_table_entry(a.v, m));
    }
};

// Row starts of U consecutive workers.  Fetched one group ahead of their use, so that with TableRows the
// pointer loads (scalar memory) overlap the previous group's row loads instead of lengthening a wave's chain
// of dependent loads.
template <typename GT, int U>
struct RowStarts {
    const GT* g[U];
    float* v[U];
};

template <typename GT, bool MOM, typename ROWS, int U>
__device__ __forceinline__ RowStarts<GT, U> fetch_rows(const StepArgs& a, int m0) {
    RowStarts<GT, U> r;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        r.g[u] = ROWS::template g<GT>(a, m0 + u);
        r.v[u] = MOM ? ROWS::v(a, m0 + u) : nullptr;
    }
    return r;
}

template <typename GT, int VEC, int SUB, bool MOM, bool OUT, bool GUARD, bool SERIAL, int U>
__device__ __forceinline__ void worker_group(const StepArgs& a, const RowStarts<GT, U>& rows, int m0, int64_t jt,
                                             uint32_t jl, const int (&nvalid)[SUB], int lane, int64_t tile0,
                                             uint32_t (&cnt)[SUB][(VEC + 1) / 2]) {
    // jt: first coordinate of the wave's first tile (wave-uniform, so row start + jt stays in scalar registers);
    // jl: this lane's offset inside a tile (32 bits).  Addresses are then "scalar base + 32-bit lane offset".
    constexpr int64_t kTile = (int64_t)kWave * VEC * kWavesPerBlock;   // a wave's tiles are a block-row apart
    // SERIAL: one row load in flight per wave.  Chosen by the launcher where momentum is written back
    // (read/write mix); the read-only forms (sign_pack, signSGD step) keep all loads of the group in flight.
    float gv[U][SUB][VEC];
    float vv[U][SUB][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int s = 0; s < SUB; ++s) {
            const GT* __restrict__ gp = (rows.g[u] + (jt + s * kTile)) + jl;       // scalar part first, then the lane's
            if constexpr (GUARD) {
                load_vals_guarded<GT, VEC>(gp, nvalid[s], gv[u][s]);
            } else {
                load_vals<VEC>(gp, gv[u][s]);
                if constexpr (SERIAL) drain_memory_ops();
            }
        }
    }
    if constexpr (MOM) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                const float* vp = (rows.v[u] + (jt + s * kTile)) + jl;
                if constexpr (GUARD) {
                    load_vals_guarded<float, VEC>(vp, nvalid[s], vv[u][s]);
                } else {
                    load_vals<VEC>(vp, vv[u][s]);
                    if constexpr (SERIAL) drain_memory_ops();
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int m = m0 + u;
        uint32_t flip = 0u;
        if constexpr (OUT) flip = a.has_flip ? ((a.flip.w[m >> 5] >> (m & 31)) & 1u) : 0u;
#pragma unroll
        for (int s = 0; s < SUB; ++s) {
            if constexpr (MOM) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    float t = a.omb * gv[u][s][c];
                    vv[u][s][c] = fmaf(a.beta, vv[u][s][c], t);
                }
                float* vp = (rows.v[u] + (jt + s * kTile)) + jl;
                if constexpr (GUARD) store_vals_guarded<float, VEC>(vp, nvalid[s], vv[u][s]);
                else store_vals<VEC>(vp, vv[u][s]);
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) vv[u][s][c] = gv[u][s][c];
            }
            uint32_t b[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                b[c] = (vv[u][s][c] >= 0.0f ? 1u : 0u) ^ flip;
                if constexpr (GUARD) b[c] = (c < nvalid[s]) ? b[c] : 0u;
                cnt[s][c >> 1] += b[c] << (16 * (c & 1));      // two 16-bit counters per register (M <= 1023)
            }
            if (OUT && a.signs_out != nullptr)
                pack_store_tile<VEC>(a.signs_out + (int64_t)m * a.signs_stride, tile0 + s * kWavesPerBlock, a.W, lane, b);
        }
    }
}

// tile0 = index of the wave's first tile of 64*VEC coordinates; its s-th tile is tile0 + 4 s
template <typename GT, typename XT, int VEC, int SUB, bool MOM, bool APPLY, bool OUT, bool GUARD, bool SERIAL,
          typename ROWS = FlatRows>
__device__ __forceinline__ void step_tiles(const StepArgs& a, int64_t tile0, int lane) {
    constexpr int64_t kTile = (int64_t)kWave * VEC * kWavesPerBlock;
    const int64_t jt = tile0 * (int64_t)(kWave * VEC);
    const uint32_t jl = (uint32_t)lane * VEC;
    const int64_t j0 = jt + jl;
    int nvalid[SUB];
#pragma unroll
    for (int s = 0; s < SUB; ++s) {
        nvalid[s] = VEC;
        if constexpr (GUARD) {
            int64_t r = a.d - (j0 + s * kTile);
            nvalid[s] = r >= VEC ? VEC : (r > 0 ? (int)r : 0);
        }
    }
    // per-coordinate counts of set sign bits, two 16-bit counters to a register: with 64 registers of row data
    // per wave the kernel sits exactly at the 96-register budget of five waves per SIMD
    uint32_t cnt[SUB][(VEC + 1) / 2];
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int c = 0; c < (VEC + 1) / 2; ++c) cnt[s][c] = 0;

    constexpr int U = 2;
    int m = 0;
    if (a.M >= U) {
        RowStarts<GT, U> cur = fetch_rows<GT, MOM, ROWS, U>(a, 0);
        for (; m + U <= a.M; m += U) {
            const int mn = (m + 2 * U <= a.M) ? m + U : m;          // the group after this one (or this one again at the end)
            const RowStarts<GT, U> nxt = fetch_rows<GT, MOM, ROWS, U>(a, mn);
            worker_group<GT, VEC, SUB, MOM, OUT, GUARD, SERIAL, U>(a, cur, m, jt, jl, nvalid, lane, tile0, cnt);
            cur = nxt;
        }
    }
    for (; m < a.M; ++m) {                                           // the M mod U workers that are left
        const RowStarts<GT, 1> last = fetch_rows<GT, MOM, ROWS, 1>(a, m);
        worker_group<GT, VEC, SUB, MOM, OUT, GUARD, SERIAL, 1>(a, last, m, jt, jl, nvalid, lane, tile0, cnt);
    }

#pragma unroll
    for (int s = 0; s < SUB; ++s) {
        uint32_t vb[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            vb[c] = (((cnt[s][c >> 1] >> (16 * (c & 1))) & 0xffffu) >= (uint32_t)a.T) ? 1u : 0u;
            if constexpr (GUARD) vb[c] = (c < nvalid[s]) ? vb[c] : 0u;
        }
        if (OUT && a.vote_out != nullptr) pack_store_tile<VEC>(a.vote_out, tile0 + s * kWavesPerBlock, a.W, lane, vb);
        if constexpr (APPLY) {
            if (nvalid[s] > 0) {
                XT* xp = (static_cast<XT*>(a.x) + (jt + s * kTile)) + jl;
                float xv[VEC];
                if constexpr (GUARD) load_vals_guarded<XT, VEC>(xp, nvalid[s], xv);
                else load_vals<VEC>(xp, xv);
#pragma unroll
                for (int c = 0; c < VEC; ++c) xv[c] = sign_update(xv[c], vb[c] != 0, a.lr, a.wd);
                if constexpr (GUARD) store_vals_guarded<XT, VEC>(xp, nvalid[s], xv);
                else store_vals<VEC>(xp, xv);
            }
        }
    }
}

// Tiles a wave of the step kernels holds at once.  4 is the measured optimum on MI355X (1 and 2 cost
// 3-8% on the resnet50-sized step).
constexpr int kStepSub = 4;

}  // namespace ssv
