// Gradient-side kernels: sign compression, worker momentum, and the whole fused iteration of
// Algorithm 1 (Signum with majority vote).  One templated kernel serves all three entry points:
//   MOM    v <- (1-beta) g + beta v  in place            (worker's momentum line)
//   sign   bit = (value >= 0), optionally flipped        (worker's send line)
//   count  per-coordinate count of set bits over the M workers, kept in registers
//          (server's sum line); vote bit = [count >= (M+1)/2]  (server's sign-of-sum line)
//   APPLY  x <- x - lr (vote + wd x)                      (the update line)
// Packed signs / packed vote are optional outputs (ballot at one coordinate per lane, a DPP
// merge of 4-bit lane groups at four).
//
// Work decomposition: a tile is 64*VEC consecutive coordinates, lane l of the wave that owns it
// holding the VEC consecutive ones at offset VEC*l, so every global access of a wave is one
// contiguous run of 16-byte (fp32) or 8-byte (bf16) lane pieces (VEC = 4; VEC = 1 is the
// any-alignment path).  A workgroup of four waves owns 4*SUB consecutive tiles, wave w holding
// tiles w, w+4, ..: the four waves' accesses of one step form one contiguous 4 KiB run per row,
// which measures about 6% faster on MI355X than giving each wave SUB adjacent tiles.
// A lane keeps its coordinates through all M workers, so nothing crosses lanes except the
// optional packing.  The kernel is HBM-bound: 12 bytes per worker-coordinate (read g, read v,
// write v) plus 8 per coordinate for x at fp32.  Per group of U = 2 workers a wave reads its
// 2*U*SUB row pieces one at a time (each load waits for the one before), then computes and issues
// the U*SUB momentum stores back to back: a read phase and a write burst per group.
#include "device_utils.h"

namespace ssv {

template <typename GT, int VEC, int SUB, bool MOM, bool OUT, bool GUARD, bool SERIAL, int U>
__device__ __forceinline__ void worker_group(const StepArgs& a, int m0, int64_t j0, const int (&nvalid)[SUB],
                                             int lane, int64_t tile0, uint32_t (&cnt)[SUB][VEC]) {
    constexpr int64_t kTile = (int64_t)kWave * VEC * kWavesPerBlock;   // a wave's tiles are a block-row apart
    // SERIAL: one row load in flight per wave.  Chosen by the launcher where momentum is written back
    // (read/write mix); the read-only forms (sign_pack, signSGD step) keep all loads of the group in flight.
    float gv[U][SUB][VEC];
    float vv[U][SUB][VEC];
    const GT* __restrict__ g = static_cast<const GT*>(a.g);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const GT* gp = g + (int64_t)(m0 + u) * a.g_stride + j0;
#pragma unroll
        for (int s = 0; s < SUB; ++s) {
            if constexpr (GUARD) {
                load_vals_guarded<GT, VEC>(gp + s * kTile, nvalid[s], gv[u][s]);
            } else {
                load_vals<VEC>(gp + s * kTile, gv[u][s]);
                if constexpr (SERIAL) drain_memory_ops();
            }
        }
    }
    if constexpr (MOM) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* vp = a.v + (int64_t)(m0 + u) * a.v_stride + j0;
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                if constexpr (GUARD) {
                    load_vals_guarded<float, VEC>(vp + s * kTile, nvalid[s], vv[u][s]);
                } else {
                    load_vals<VEC>(vp + s * kTile, vv[u][s]);
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
                float* vp = a.v + (int64_t)m * a.v_stride + j0 + s * kTile;
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
                cnt[s][c] += b[c];
            }
            if (OUT && a.signs_out != nullptr)
                pack_store_tile<VEC>(a.signs_out + (int64_t)m * a.signs_stride, tile0 + s * kWavesPerBlock, a.W, lane, b);
        }
    }
}

// tile0 = index of the wave's first tile of 64*VEC coordinates; its s-th tile is tile0 + 4 s
template <typename GT, typename XT, int VEC, int SUB, bool MOM, bool APPLY, bool OUT, bool GUARD, bool SERIAL>
__device__ __forceinline__ void step_tiles(const StepArgs& a, int64_t tile0, int lane) {
    constexpr int64_t kTile = (int64_t)kWave * VEC * kWavesPerBlock;
    const int64_t j0 = tile0 * (int64_t)(kWave * VEC) + (int64_t)lane * VEC;
    int nvalid[SUB];
#pragma unroll
    for (int s = 0; s < SUB; ++s) {
        nvalid[s] = VEC;
        if constexpr (GUARD) {
            int64_t r = a.d - (j0 + s * kTile);
            nvalid[s] = r >= VEC ? VEC : (r > 0 ? (int)r : 0);
        }
    }
    uint32_t cnt[SUB][VEC];
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int c = 0; c < VEC; ++c) cnt[s][c] = 0;

    constexpr int U = 2;
    int m = 0;
    for (; m + U <= a.M; m += U)
        worker_group<GT, VEC, SUB, MOM, OUT, GUARD, SERIAL, U>(a, m, j0, nvalid, lane, tile0, cnt);
    if (m < a.M) worker_group<GT, VEC, SUB, MOM, OUT, GUARD, SERIAL, 1>(a, m, j0, nvalid, lane, tile0, cnt);

#pragma unroll
    for (int s = 0; s < SUB; ++s) {
        uint32_t vb[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            vb[c] = (cnt[s][c] >= (uint32_t)a.T) ? 1u : 0u;
            if constexpr (GUARD) vb[c] = (c < nvalid[s]) ? vb[c] : 0u;
        }
        if (OUT && a.vote_out != nullptr) pack_store_tile<VEC>(a.vote_out, tile0 + s * kWavesPerBlock, a.W, lane, vb);
        if constexpr (APPLY) {
            if (nvalid[s] > 0) {
                XT* xp = static_cast<XT*>(a.x) + j0 + s * kTile;
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

// Blocks 0 .. nfull-1 each take 4*SUB consecutive tiles: in step s (s < SUB) the block's four waves
// touch four adjacent tiles, i.e. one contiguous 4 KiB run of every row.  The waves of the blocks
// after them take the remaining (fewer than 4*SUB + 1) tiles one by one with bounds checks.
// OUT = false is the lean form without optional outputs (packed signs, packed vote, flips).
template <typename GT, typename XT, int VEC, int SUB, bool MOM, bool APPLY, bool OUT, bool SERIAL>
__global__ __launch_bounds__(kBlock) void step_kernel(StepArgs a, int64_t nfull) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t lb = blockIdx.x;
    if (lb < nfull) {
        step_tiles<GT, XT, VEC, SUB, MOM, APPLY, OUT, false, SERIAL>(a, lb * (kWavesPerBlock * SUB) + wave, lane);
    } else {
        const int64_t tile = nfull * (kWavesPerBlock * SUB) + (lb - nfull) * kWavesPerBlock + wave;
        if (tile < a.ntiles) step_tiles<GT, XT, VEC, 1, MOM, APPLY, OUT, true, false>(a, tile, lane);
    }
}

// Tiles a wave of the step kernel holds at once.  4 is the measured optimum on MI355X (1 and 2 cost
// 3-8% on the resnet50-sized step).
constexpr int kStepSub = 4;

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY, bool OUT, bool SERIAL>
static hipError_t launch_out(StepArgs a, hipStream_t s) {
    constexpr int SUB = kStepSub;
    constexpr int64_t kTile = (int64_t)kWave * VEC;
    constexpr int64_t kBlockTiles = (int64_t)kWavesPerBlock * SUB;
    a.ntiles = (a.d + kTile - 1) / kTile;
    const int64_t nfull = a.d / (kTile * kBlockTiles);
    const int64_t tail_tiles = a.ntiles - nfull * kBlockTiles;
    const int64_t grid = nfull + (tail_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((step_kernel<GT, XT, VEC, SUB, MOM, APPLY, OUT, SERIAL>), dim3((unsigned)grid), dim3(kBlock), 0,
                       s, a, nfull);
    return hipGetLastError();
}

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY, bool OUT>
static hipError_t launch_serial(const StepArgs& a, hipStream_t s) {
    // One row load in flight per wave where the kernel also writes momentum back (see drain_memory_ops);
    // SSV_TUNE_STEP_SERIAL=0 switches that off for A/B measurements.
    if constexpr (MOM && VEC > 1) {
        if (tuning().step_serial) return launch_out<GT, XT, VEC, MOM, APPLY, OUT, true>(a, s);
    }
    return launch_out<GT, XT, VEC, MOM, APPLY, OUT, false>(a, s);
}

template <typename GT, typename XT, int VEC, bool MOM, bool APPLY>
static hipError_t launch_one(const StepArgs& a, hipStream_t s) {
    const bool out = a.signs_out != nullptr || a.vote_out != nullptr || a.has_flip;
    if constexpr (!APPLY) return launch_serial<GT, XT, VEC, MOM, APPLY, true>(a, s);   // pack-only forms
    else return out ? launch_serial<GT, XT, VEC, MOM, APPLY, true>(a, s)
                    : launch_serial<GT, XT, VEC, MOM, APPLY, false>(a, s);
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
    // bf16 gradients also use 4 coordinates per lane (8-byte g pieces, 16-byte v pieces): every
    // momentum access of a wave is then one contiguous KiB.  With 8 per lane the two 16-byte v
    // pieces of a lane interleave with its neighbours' and the step runs at 65% instead of 76%.
    return vector_ok ? launch_g<bf16, 4>(a, x_dt, s) : launch_g<bf16, 1>(a, x_dt, s);
}

}  // namespace ssv
