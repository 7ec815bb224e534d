// Gradient-side kernels: sign compression, worker momentum, and the whole fused iteration of
// Algorithm 1 ("Signum with majority vote").  One templated kernel serves all three entry points:
//   MOM    v <- (1-beta) g + beta v  in place            ("update momentum")
//   sign   bit = (value >= 0), optionally flipped        ("push sign(v_m)")
//   count  per-coordinate count of set bits over the M workers, kept in registers
//          ("aggregate sign momenta"); vote bit = [count >= (M+1)/2]
//   APPLY  x <- x - lr (vote + wd x)                      ("update parameters")
// Packed signs / packed vote are optional outputs built with wave ballots.
//
// Work decomposition: a wavefront owns a tile of 64*VEC consecutive coordinates, lane l owning the
// VEC consecutive ones at 64*VEC*tile + VEC*l, so that every global access of a wave is one
// contiguous run of 16-byte lane pieces (VEC = 4 for fp32 gradients, 8 for bf16; VEC = 1 is the
// any-alignment path).  A lane keeps its coordinates through all M workers, so nothing crosses
// lanes except the optional ballots.  The kernel is HBM-bound: 12 bytes per worker-coordinate
// (read g, read v, write v) plus 8 per coordinate for x at fp32.
#include "device_utils.h"

namespace ssv {

template <typename GT, int VEC, bool MOM, bool GUARD, int U>
__device__ __forceinline__ void worker_group(const StepArgs& a, int m0, int64_t j0, int nvalid, int lane,
                                             int64_t tile, uint32_t (&cnt)[VEC]) {
    float gv[U][VEC];
    float vv[U][VEC];
    const GT* __restrict__ g = static_cast<const GT*>(a.g);
    // all loads of the group first, so that up to 2*U 16-byte loads per lane are in flight
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const GT* gp = g + (int64_t)(m0 + u) * a.g_stride + j0;
        if constexpr (GUARD) load_vals_guarded<GT, VEC>(gp, nvalid, gv[u]);
        else load_vals<VEC>(gp, gv[u]);
    }
    if constexpr (MOM) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* vp = a.v + (int64_t)(m0 + u) * a.v_stride + j0;
            if constexpr (GUARD) load_vals_guarded<float, VEC>(vp, nvalid, vv[u]);
            else load_vals<VEC>(vp, vv[u]);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int m = m0 + u;
        if constexpr (MOM) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                float t = a.omb * gv[u][c];
                vv[u][c] = fmaf(a.beta, vv[u][c], t);
            }
            float* vp = a.v + (int64_t)m * a.v_stride + j0;
            if constexpr (GUARD) store_vals_guarded<float, VEC>(vp, nvalid, vv[u]);
            else store_vals<VEC>(vp, vv[u]);
        } else {
#pragma unroll
            for (int c = 0; c < VEC; ++c) vv[u][c] = gv[u][c];
        }
        const uint32_t flip = a.has_flip ? ((a.flip.w[m >> 5] >> (m & 31)) & 1u) : 0u;
        uint32_t b[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            b[c] = (vv[u][c] >= 0.0f ? 1u : 0u) ^ flip;
            if constexpr (GUARD) b[c] = (c < nvalid) ? b[c] : 0u;
            cnt[c] += b[c];
        }
        if (a.signs_out != nullptr) {
            uint64_t words[VEC];
            pack_tile<VEC>(b, words);
            store_tile_words<VEC>(a.signs_out + (int64_t)m * a.signs_stride, tile, a.W, lane, words);
        }
    }
}

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY, bool GUARD>
__device__ __forceinline__ void step_tile(const StepArgs& a, int64_t tile, int lane) {
    const int64_t j0 = tile * (int64_t)(kWave * VEC) + (int64_t)lane * VEC;
    int nvalid = VEC;
    if constexpr (GUARD) {
        int64_t r = a.d - j0;
        nvalid = r >= VEC ? VEC : (r > 0 ? (int)r : 0);
    }
    uint32_t cnt[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) cnt[c] = 0;

    constexpr int U = (VEC >= 8) ? 2 : 4;      // keeps 8 sixteen-byte loads per lane in flight
    int m = 0;
    for (; m + U <= a.M; m += U) worker_group<GT, VEC, MOM, GUARD, U>(a, m, j0, nvalid, lane, tile, cnt);
    if constexpr (U == 4) {
        if (m + 2 <= a.M) { worker_group<GT, VEC, MOM, GUARD, 2>(a, m, j0, nvalid, lane, tile, cnt); m += 2; }
    }
    if (m < a.M) worker_group<GT, VEC, MOM, GUARD, 1>(a, m, j0, nvalid, lane, tile, cnt);

    uint32_t vb[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        vb[c] = (cnt[c] >= (uint32_t)a.T) ? 1u : 0u;
        if constexpr (GUARD) vb[c] = (c < nvalid) ? vb[c] : 0u;
    }
    if (a.vote_out != nullptr) {
        uint64_t words[VEC];
        pack_tile<VEC>(vb, words);
        store_tile_words<VEC>(a.vote_out, tile, a.W, lane, words);
    }
    if constexpr (APPLY) {
        if (nvalid > 0) {
            XT* xp = static_cast<XT*>(a.x) + j0;
            float xv[VEC];
            if constexpr (GUARD) load_vals_guarded<XT, VEC>(xp, nvalid, xv);
            else load_vals<VEC>(xp, xv);
#pragma unroll
            for (int c = 0; c < VEC; ++c) xv[c] = sign_update(xv[c], vb[c] != 0, a.lr, a.wd);
            if constexpr (GUARD) store_vals_guarded<XT, VEC>(xp, nvalid, xv);
            else store_vals<VEC>(xp, xv);
        }
    }
}

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY>
__global__ __launch_bounds__(kBlock) void step_kernel(StepArgs a, int tiles_per_wave, int64_t nblocks,
                                                      int remap) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t lb = logical_block(blockIdx.x, nblocks, remap);
    if (lb >= nblocks) return;
    const int64_t tile0 = lb * (int64_t)(kWavesPerBlock * tiles_per_wave) + wave;
    for (int t = 0; t < tiles_per_wave; ++t) {
        const int64_t tile = tile0 + (int64_t)t * kWavesPerBlock;
        if (tile >= a.ntiles) break;
        if ((tile + 1) * (int64_t)(kWave * VEC) <= a.d)
            step_tile<GT, XT, VEC, MOM, APPLY, false>(a, tile, lane);
        else
            step_tile<GT, XT, VEC, MOM, APPLY, true>(a, tile, lane);
    }
}

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY>
static hipError_t launch_one(StepArgs a, hipStream_t s) {
    const Tuning& tn = tuning();
    a.ntiles = (a.d + (int64_t)kWave * VEC - 1) / ((int64_t)kWave * VEC);
    int tpw = tn.step_tiles_per_wave > 0 ? tn.step_tiles_per_wave : 1;
    int64_t tiles_per_block = (int64_t)kWavesPerBlock * tpw;
    int64_t nblocks = (a.ntiles + tiles_per_block - 1) / tiles_per_block;
    int64_t grid = tn.xcd_remap ? 8 * ((nblocks + 7) / 8) : nblocks;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((step_kernel<GT, XT, VEC, MOM, APPLY>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, tpw,
                       nblocks, tn.xcd_remap);
    return hipGetLastError();
}

template <typename GT, int VEC>
static hipError_t launch_g(const StepArgs& a, int x_dt, hipStream_t s) {
    const bool mom = a.v != nullptr;
    const bool apply = a.x != nullptr;
    if (!apply) {
        return mom ? launch_one<GT, float, VEC, true, false>(a, s) : launch_one<GT, float, VEC, false, false>(a, s);
    }
    if (x_dt == 0) {
        return mom ? launch_one<GT, float, VEC, true, true>(a, s) : launch_one<GT, float, VEC, false, true>(a, s);
    }
    return mom ? launch_one<GT, bf16, VEC, true, true>(a, s) : launch_one<GT, bf16, VEC, false, true>(a, s);
}

hipError_t launch_step(const StepArgs& a, int g_dt, int x_dt, bool vector_ok, hipStream_t s) {
    if (g_dt == 0) return vector_ok ? launch_g<float, 4>(a, x_dt, s) : launch_g<float, 1>(a, x_dt, s);
    return vector_ok ? launch_g<bf16, 8>(a, x_dt, s) : launch_g<bf16, 1>(a, x_dt, s);
}

}  // namespace ssv
