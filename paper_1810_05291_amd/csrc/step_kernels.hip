// Gradient-side kernels: sign compression, worker momentum, and the whole iteration of Algorithm 1 (Signum with
// majority vote) fused into one kernel.
//   MOM    v <- (1-beta) g + beta v  in place            (worker's momentum line)
//   sign   bit = (value >= 0), optionally flipped        (worker's send line)
//   count  per-coordinate count of set bits over the M workers, kept in registers
//          (server's sum line); vote bit = [count >= (M+1)/2]  (server's sign-of-sum line)
//   update x <- x - lr (vote + wd x)                      (the update line)
// Packed signs / packed vote are optional outputs (ballot at one coordinate per lane, a DPP merge of 4-bit lane
// groups at four).
//
// Two kernels share the tile body (step_tiles.h):
//   step_kernel       all of the above in one pass; a workgroup walks all M rows of its tiles.  Signs and counts
//                     never leave registers.  Serves ssv_signum_step when the caller gives no room for packed signs.
//   pack_rows_kernel  momentum + sign + pack of ONE row per workgroup, grid (tile groups) x (workers).  Serves
//                     ssv_sign_pack, ssv_signum_momentum_pack, and the first half of ssv_signum_step when the caller
//                     provides `signs_out` (the packed vote + update kernel of vote_kernels.hip is the second half).
// On MI355X the second, row-by-row form sustains 83% of the HBM peak and the first 75% (M = 15; 72% at M = 31),
// although the first moves 2% fewer bytes: what the memory system rewards is few, compact streams.
//
// Work decomposition: a tile is 64*VEC consecutive coordinates, lane l of the wave that owns it holding the VEC
// consecutive ones at offset VEC*l, so every global access of a wave is one contiguous run of 16-byte (fp32) or
// 8-byte (bf16) lane pieces (VEC = 4; VEC = 1 is the any-alignment path).  A workgroup of four waves owns 4*SUB
// consecutive tiles, wave w holding tiles w, w+4, ..: the four waves' accesses of one step form one contiguous
// 4 KiB run per row, which measures about 6% faster than giving each wave SUB adjacent tiles.  Both kernels are
// HBM-bound: 12 bytes per worker-coordinate (read g, read v, write v) plus 8 per coordinate for x at fp32.
#include "step_tiles.h"

namespace ssv {

constexpr int64_t kShortVector = int64_t(1) << 21;      // coordinates below which the one-kernel step uses 1 tile per wave

// ---- the one-kernel step --------------------------------------------------------------------------------------
// Per group of U = 2 workers a wave reads its 2*U*SUB row pieces one at a time (each load waits for the one before),
// then computes and issues the U*SUB momentum stores back to back: a read phase and a write burst per group.
// Blocks 0 .. nfull-1 each take 4*SUB consecutive tiles: in step s (s < SUB) the block's four waves
// touch four adjacent tiles, i.e. one contiguous 4 KiB run of every row.  The waves of the blocks
// after them take the remaining (fewer than 4*SUB + 1) tiles one by one with bounds checks.
// OUT = false is the lean form without optional outputs (packed signs, packed vote, flips).
template <typename GT, typename XT, int VEC, int SUB, bool MOM, bool OUT, bool SERIAL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(5, 5))) void step_kernel(StepArgs a, int64_t nfull) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);      // tell the compiler it is wave-uniform
    const int64_t lb = blockIdx.x;
    if (lb < nfull) {
        step_tiles<GT, XT, VEC, SUB, MOM, true, OUT, false, SERIAL>(a, lb * (kWavesPerBlock * SUB) + wave, lane);
    } else {
        const int64_t tile = nfull * (kWavesPerBlock * SUB) + (lb - nfull) * kWavesPerBlock + wave;
        if (tile < a.ntiles) step_tiles<GT, XT, VEC, 1, MOM, true, OUT, true, false>(a, tile, lane);
    }
}

template <typename GT, typename XT, int VEC, bool MOM, bool OUT, bool SERIAL, int SUB = kStepSub>
static hipError_t launch_out(StepArgs a, hipStream_t s) {
    // Short vectors: with fewer than about 500 workgroups of 16 tiles the chip is not full and every wave walks a
    // long chain of dependent loads, so such calls use one tile per wave (four times the workgroups, a quarter of
    // the chain).  M = 15: d = 2^20 69 -> 33 us, d = 2^16 57 -> 17 us; from d = 2^22 on the 4-tile form is faster.
    if constexpr (SUB == kStepSub) {
        if (a.d < kShortVector) return launch_out<GT, XT, VEC, MOM, OUT, SERIAL, 1>(a, s);
    }
    constexpr int64_t kTile = (int64_t)kWave * VEC;
    constexpr int64_t kBlockTiles = (int64_t)kWavesPerBlock * SUB;
    a.ntiles = (a.d + kTile - 1) / kTile;
    const int64_t nfull = a.d / (kTile * kBlockTiles);
    const int64_t tail_tiles = a.ntiles - nfull * kBlockTiles;
    const int64_t grid = nfull + (tail_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((step_kernel<GT, XT, VEC, SUB, MOM, OUT, SERIAL>), dim3((unsigned)grid), dim3(kBlock), 0,
                       s, a, nfull);
    return hipGetLastError();
}

// ---- pack-only forms: ssv_sign_pack, ssv_signum_momentum_pack, first half of the two-kernel step ---------------
// Grid (tile groups, M): a workgroup handles 4*SUB consecutive tiles of ONE row (wave w tiles w, w+4, ..), and the
// workgroups of row m are all handed out before those of row m+1.  At any moment the whole chip therefore works on
// a window of a few MiB that slides along one or two rows: three compact streams (g_m, v_m in, v_m out) instead of
// the 2M+1 streams of step_kernel.  Measured on the resnet50-sized momentum+pack (M = 15 / 31): 83% of the HBM peak
// for both, against 76% / 73% with the M rows looped over inside each workgroup, and 79% against 72% for the
// sign-only form.  What does NOT work is to give each resident workgroup a private range to sweep row after
// row (a persistent grid): every stream then has as many scattered access points as there are workgroups (66%).
//   momentum form: SUB = 1, one row load in flight per wave (load g, load v, store v: SUB = 2 / 4 / 8 measured
//                  79 / 75 / 72%), as many waves per SIMD as fit (capping them at 5 costs 17 points);
//   sign-only form: SUB = 4 with all loads in flight (SUB = 1 / 2 / 8: 72 / 75 / 77%).
// The rows' ragged ends are taken by the workgroups behind the first nfat of each row, tile by tile with bounds checks.
template <typename GT, int VEC, int SUB, bool MOM, bool SERIAL>
__global__ __launch_bounds__(kBlock) void pack_rows_kernel(StepArgs a, int64_t nfat) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);      // tell the compiler it is wave-uniform
    const int m = blockIdx.y;
    const int64_t lb = blockIdx.x;
    constexpr int64_t kTileCoords = (int64_t)kWave * VEC;
    const RowStarts<GT, 1> row = fetch_rows<GT, MOM, FlatRows, 1>(a, m);
    const uint32_t jl = (uint32_t)lane * VEC;
    if (lb < nfat) {
        const int64_t tile0 = lb * (kWavesPerBlock * SUB) + wave;
        int nvalid[SUB];
        uint32_t unused_count[SUB][(VEC + 1) / 2];                // worker_group counts set bits for the vote: dead code here
#pragma unroll
        for (int q = 0; q < SUB; ++q) {
            nvalid[q] = VEC;
#pragma unroll
            for (int c = 0; c < (VEC + 1) / 2; ++c) unused_count[q][c] = 0;
        }
        worker_group<GT, VEC, SUB, MOM, true, false, SERIAL, 1>(a, row, m, tile0 * kTileCoords, jl, nvalid, lane, tile0,
                                                                unused_count);
    } else {
        const int64_t tile = nfat * (kWavesPerBlock * SUB) + (lb - nfat) * kWavesPerBlock + wave;
        if (tile < a.ntiles) {                                     // wave-uniform
            const int64_t left = a.d - (tile * kTileCoords + jl);
            int nvalid[1] = {left >= VEC ? VEC : (left > 0 ? (int)left : 0)};
            uint32_t unused_count[1][(VEC + 1) / 2] = {};
            worker_group<GT, VEC, 1, MOM, true, true, false, 1>(a, row, m, tile * kTileCoords, jl, nvalid, lane, tile,
                                                                unused_count);
        }
    }
}

template <typename GT, int VEC, int SUB, bool MOM, bool SERIAL>
static hipError_t launch_pack_rows(StepArgs a, hipStream_t s) {
    constexpr int64_t kTile = (int64_t)kWave * VEC;
    constexpr int64_t kBlockTiles = (int64_t)kWavesPerBlock * SUB;
    a.ntiles = (a.d + kTile - 1) / kTile;
    const int64_t nfat = (a.d / kTile) / kBlockTiles;
    const int64_t tail_tiles = a.ntiles - nfat * kBlockTiles;
    const int64_t grid = nfat + (tail_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (grid > 0x7fffffffLL || a.M > 65535) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    hipLaunchKernelGGL((pack_rows_kernel<GT, VEC, SUB, MOM, SERIAL>), dim3((unsigned)grid, (unsigned)a.M), dim3(kBlock), 0,
                       s, a, nfat);
    return hipGetLastError();
}

template <typename GT, int VEC>
static hipError_t launch_pack(const StepArgs& a, hipStream_t s) {
    if (a.v != nullptr) {
        // SSV_TUNE_STEP_SERIAL=0 lets both loads of a tile go out together (A/B measurements)
        return tuning().step_serial ? launch_pack_rows<GT, VEC, 1, true, true>(a, s)
                                    : launch_pack_rows<GT, VEC, 1, true, false>(a, s);
    }
    return launch_pack_rows<GT, VEC, 4, false, false>(a, s);
}

template <typename GT, typename XT, int VEC, bool MOM, bool OUT>
static hipError_t launch_serial(const StepArgs& a, hipStream_t s) {
    // One row load in flight per wave where the kernel also writes momentum back (see drain_memory_ops);
    // SSV_TUNE_STEP_SERIAL=0 switches that off for A/B measurements.
    if constexpr (MOM && VEC > 1) {
        if (tuning().step_serial) return launch_out<GT, XT, VEC, MOM, OUT, true>(a, s);
    }
    return launch_out<GT, XT, VEC, MOM, OUT, false>(a, s);
}

template <typename GT, typename XT, int VEC, bool MOM>
static hipError_t launch_one(const StepArgs& a, hipStream_t s) {
    const bool out = a.signs_out != nullptr || a.vote_out != nullptr || a.has_flip;
    return out ? launch_serial<GT, XT, VEC, MOM, true>(a, s) : launch_serial<GT, XT, VEC, MOM, false>(a, s);
}

template <typename GT, int VEC>
static hipError_t launch_g(const StepArgs& a, int x_dt, hipStream_t s) {
    const bool mom = a.v != nullptr;
    if (a.x == nullptr) return launch_pack<GT, VEC>(a, s);          // no update: the pack-only forms
    if (x_dt == 0) {
        return mom ? launch_one<GT, float, VEC, true>(a, s) : launch_one<GT, float, VEC, false>(a, s);
    }
    return mom ? launch_one<GT, bf16, VEC, true>(a, s) : launch_one<GT, bf16, VEC, false>(a, s);
}

hipError_t launch_step(const StepArgs& a, int g_dt, int x_dt, bool vector_ok, hipStream_t s) {
    if (g_dt == 0) return vector_ok ? launch_g<float, 4>(a, x_dt, s) : launch_g<float, 1>(a, x_dt, s);
    // bf16 gradients also use 4 coordinates per lane (8-byte g pieces, 16-byte v pieces): every
    // momentum access of a wave is then one contiguous KiB.  With 8 per lane the two 16-byte v
    // pieces of a lane interleave with its neighbours' and the step runs at 65% instead of 76%.
    return vector_ok ? launch_g<bf16, 4>(a, x_dt, s) : launch_g<bf16, 1>(a, x_dt, s);
}

}  // namespace ssv
