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
#include "step_tiles.h"

namespace ssv {

// Blocks 0 .. nfull-1 each take 4*SUB consecutive tiles: in step s (s < SUB) the block's four waves
// touch four adjacent tiles, i.e. one contiguous 4 KiB run of every row.  The waves of the blocks
// after them take the remaining (fewer than 4*SUB + 1) tiles one by one with bounds checks.
// OUT = false is the lean form without optional outputs (packed signs, packed vote, flips).
template <typename GT, typename XT, int VEC, int SUB, bool MOM, bool APPLY, bool OUT, bool SERIAL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(5, 5))) void step_kernel(StepArgs a, int64_t nfull) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);      // tell the compiler it is wave-uniform
    const int64_t lb = blockIdx.x;
    if (lb < nfull) {
        step_tiles<GT, XT, VEC, SUB, MOM, APPLY, OUT, false, SERIAL>(a, lb * (kWavesPerBlock * SUB) + wave, lane);
    } else {
        const int64_t tile = nfull * (kWavesPerBlock * SUB) + (lb - nfull) * kWavesPerBlock + wave;
        if (tile < a.ntiles) step_tiles<GT, XT, VEC, 1, MOM, APPLY, OUT, true, false>(a, tile, lane);
    }
}

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
