// Ternary QSGD (the comparison compressors of Appendix B): per-row norms, the stochastic ternary choice packed
// into two bit planes, and the 1-way average fused with the SGD update.  C ABI in include/signvote_qsgd.h.
//
// All three kernels are HBM-bound streams:
//   norms      4 B read per worker-coordinate (2 for bf16); per-lane double accumulators, a fixed reduction
//              order (lane -> wavefront -> workgroup -> one partial per workgroup in the workspace -> a finishing
//              kernel that adds the partials of a row in index order), so results do not vary from run to run
//   quantize   8 B read (g and u) and 2 bits written per worker-coordinate; packing as for the sign vectors
//   aggregate  2 M bits read and 4 / 8 / 12 B moved per coordinate (avg_out and / or x); the per-lane sums are
//              handed over through LDS so that the plane reads and the weight accesses are both contiguous
#include <cmath>
#include <mutex>

#include "../../include/signvote.h"
#include "../../include/signvote_qsgd.h"
#include "device_utils.h"

namespace ssv {

constexpr int kNormParts = 256;          // workgroups (= partial results) per row in the norm kernel
constexpr int kNormUnroll = 4;           // independent 16-byte loads per lane per round

struct NormArgs {
    const void* g;
    double* partial;        // [M][kNormParts]
    float* norms;           // [M]
    int64_t d, g_stride;
    int M, kind;
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off, kWave));
    return v;
}

// Workgroup (p, m) walks row m in rounds of kNormParts * 256 * VEC * kNormUnroll coordinates.
template <typename GT, int VEC, bool L2>
__global__ __launch_bounds__(kBlock) void qsgd_norm_partial_kernel(NormArgs a) {
    __shared__ double wave_part[kWavesPerBlock];
    const int m = blockIdx.y;
    const GT* __restrict__ row = static_cast<const GT*>(a.g) + (int64_t)m * a.g_stride;
    constexpr int64_t kChunk = (int64_t)kBlock * VEC;                       // coordinates per workgroup access
    const int64_t round = (int64_t)kNormParts * kChunk * kNormUnroll;
    double acc = 0.0;
    for (int64_t base = (int64_t)blockIdx.x * kChunk * kNormUnroll; base < a.d; base += round) {
        float gv[kNormUnroll][VEC];
#pragma unroll
        for (int k = 0; k < kNormUnroll; ++k) {
            const int64_t j = base + k * kChunk + (int64_t)threadIdx.x * VEC;
            const int64_t left = a.d - j;
            const int n = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
            if (n > 0) {
                load_vals_guarded<GT, VEC>(row + j, n, gv[k]);              // elements past the end read as 0
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) gv[k][c] = 0.0f;
            }
        }
#pragma unroll
        for (int k = 0; k < kNormUnroll; ++k)
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const double x = (double)gv[k][c];
                if constexpr (L2) acc += x * x;                             // the square of an fp32 number is exact in double
                else acc = fmax(acc, fabs(x));                              // fmax returns the number when one side is NaN
            }
    }
    acc = L2 ? wave_sum(acc) : wave_max(acc);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) wave_part[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double r = wave_part[0];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) r = L2 ? r + wave_part[w] : fmax(r, wave_part[w]);
        a.partial[(int64_t)m * kNormParts + blockIdx.x] = r;
    }
}

// One workgroup per row: thread p holds partial p.
template <bool L2>
__global__ __launch_bounds__(kBlock) void qsgd_norm_finish_kernel(NormArgs a) {
    static_assert(kNormParts == kBlock, "one partial per thread");
    __shared__ double wave_part[kWavesPerBlock];
    const int m = blockIdx.x;
    double v = a.partial[(int64_t)m * kNormParts + threadIdx.x];
    v = L2 ? wave_sum(v) : wave_max(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) wave_part[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        double r = wave_part[0];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) r = L2 ? r + wave_part[w] : fmax(r, wave_part[w]);
        a.norms[m] = (float)(L2 ? sqrt(r) : r);
    }
}

// ---- quantise ---------------------------------------------------------------------------------------------
struct QuantArgs {
    const void* g;
    const float* u;
    const float* norms;
    uint64_t* nonzero;
    uint64_t* sign;
    int64_t d, g_stride, u_stride, words_stride, W;
};

template <typename GT, int VEC, bool GUARD>
__device__ __forceinline__ void quant_tile(const QuantArgs& a, const GT* __restrict__ grow, const float* __restrict__ urow,
                                           float norm, uint64_t* nzrow, uint64_t* sgrow, int64_t tile, int lane) {
    const int64_t j0 = tile * (int64_t)(kWave * VEC) + (int64_t)lane * VEC;
    int n = VEC;
    if constexpr (GUARD) {
        const int64_t left = a.d - j0;
        n = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
    }
    float gv[VEC], uv[VEC];
    if constexpr (GUARD) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) { gv[c] = 0.0f; uv[c] = 0.0f; }
        if (n > 0) {
            load_vals_guarded<GT, VEC>(grow + j0, n, gv);
            load_vals_guarded<float, VEC>(urow + j0, n, uv);
        }
    } else {
        load_vals<VEC>(grow + j0, gv);
        load_vals<VEC>(urow + j0, uv);
    }
    uint32_t nzb[VEC], sgb[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        const float threshold = uv[c] * norm;
        const bool keep = (threshold < fabsf(gv[c])) && (!GUARD || c < n);
        nzb[c] = keep ? 1u : 0u;
        sgb[c] = (keep && gv[c] > 0.0f) ? 1u : 0u;
    }
    // every lane of the wave reaches both calls (cross-lane merge of the 4-bit groups)
    pack_store_tile<VEC>(nzrow, tile, a.W, lane, nzb);
    pack_store_tile<VEC>(sgrow, tile, a.W, lane, sgb);
}

// Workgroup (b, m): 4 * kQuantSub consecutive tiles of row m, wave w holding tiles w, w+4, ..; the ragged last
// workgroup of a row walks its tiles with bounds checks.  Rows are handed out one after the other, so the chip
// reads a compact window of two streams (g_m and u_m) at a time; one tile per wave measured best on MI355X
// (resnet50 size, M = 15: 1 / 2 / 4 / 8 tiles per wave = 80.7 / 77.8 / 76.0 / 74.5% of the HBM peak).
constexpr int kQuantSub = 1;
template <typename GT, int VEC>
__global__ __launch_bounds__(kBlock) void qsgd_quantize_kernel(QuantArgs a, int64_t nfull, int64_t ntiles) {
    constexpr int SUB = kQuantSub;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int m = blockIdx.y;
    const GT* __restrict__ grow = static_cast<const GT*>(a.g) + (int64_t)m * a.g_stride;
    const float* __restrict__ urow = a.u + (int64_t)m * a.u_stride;
    uint64_t* nzrow = a.nonzero + (int64_t)m * a.words_stride;
    uint64_t* sgrow = a.sign + (int64_t)m * a.words_stride;
    const float norm = a.norms[m];
    const int64_t tile0 = (int64_t)blockIdx.x * (kWavesPerBlock * SUB) + wave;
    if ((int64_t)blockIdx.x < nfull) {
#pragma unroll
        for (int s = 0; s < SUB; ++s)
            quant_tile<GT, VEC, false>(a, grow, urow, norm, nzrow, sgrow, tile0 + s * kWavesPerBlock, lane);
    } else {
        for (int s = 0; s < SUB; ++s) {
            const int64_t tile = tile0 + s * kWavesPerBlock;
            if (tile < ntiles) quant_tile<GT, VEC, true>(a, grow, urow, norm, nzrow, sgrow, tile, lane);   // wave-uniform
        }
    }
}

// ---- 1-way average + update -------------------------------------------------------------------------------
typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));

struct AggArgs {
    const uint64_t* nonzero;
    const uint64_t* sign;
    const float* norms;
    float* avg_out;
    void* x;
    int64_t d, words_stride;
    int M;
    float inv_m, lr;
};

// A wavefront owns a tile of 2048 coordinates = 64 dwords of every plane row.  Lane l loads dword l of both planes
// for every worker (two 256-byte reads per worker per wave) and sums the decoded values of ITS 32 coordinates in 32
// registers, workers in index order.  Decoding goes through a 256-entry table in LDS: the 4 nonzero bits and 4 sign
// bits of four neighbouring coordinates index a float4 of {0, +1, -1} factors, and acc <- fma(norm, factor, acc)
// adds +norm, -norm or +0 exactly (norm finite; a worker whose norm is Inf or NaN takes a mask-based path, because
// Inf * 0 is not 0).  That is about 1.6 vector operations per worker-coordinate.  Earlier forms: a lane reading
// the plane BYTE of its 4 coordinates per worker was bound by the number of load instructions (25% of the HBM
// peak); "acc = keep ? acc +- norm : acc" compiles to compares and EXEC-mask juggling (39%); one-bit signed
// bit-field extracts and masks take 5 operations per worker-coordinate, which at M = 15 is more ALU time than the
// kernel's HBM time (55%).
// The averages then change hands through LDS (a padded per-wave array, no bank conflicts) so that the weight /
// average accesses are contiguous: lane l takes elements (i * 64 + l) * VEC of the tile in access i.
template <typename XT, int VEC>
__global__ __launch_bounds__(kBlock) void qsgd_aggregate_kernel(AggArgs a, int64_t ntiles) {
    constexpr int kTileCoords = kWave * 32;
    constexpr int kPad = 33;                                        // row pitch of a lane's 32 values: odd => conflict-free
    __shared__ float stage[kWavesPerBlock][kWave * kPad];
    __shared__ h16x4 factor[256];                                   // {0, +1, -1} are exact in half precision
    {
        const uint32_t i = threadIdx.x;                             // kBlock == 256: one table entry per thread
        h16x4 q;
        q.x = (_Float16)((i & 1u) ? ((i & 16u) ? 1.0f : -1.0f) : 0.0f);
        q.y = (_Float16)((i & 2u) ? ((i & 32u) ? 1.0f : -1.0f) : 0.0f);
        q.z = (_Float16)((i & 4u) ? ((i & 64u) ? 1.0f : -1.0f) : 0.0f);
        q.w = (_Float16)((i & 8u) ? ((i & 128u) ? 1.0f : -1.0f) : 0.0f);
        factor[i] = q;
    }
    __syncthreads();                                                // every thread of the workgroup reaches this
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    if (tile >= ntiles) return;                                     // wave-uniform; no workgroup barrier below
    const int64_t W2 = 2 * ((a.d + 63) / 64);                       // dwords per plane row that exist
    const int64_t dw = tile * kWave + lane;
    const bool have = dw < W2;
    const int64_t row_dw = 2 * a.words_stride;
    const uint32_t* __restrict__ nzp = reinterpret_cast<const uint32_t*>(a.nonzero) + dw;
    const uint32_t* __restrict__ sgp = reinterpret_cast<const uint32_t*>(a.sign) + dw;
    const int64_t cbase = tile * (int64_t)kTileCoords;
    const int64_t left = a.d - cbase;                               // > 0
    const bool full = left >= kTileCoords;                          // wave-uniform
    constexpr int kAcc = 32 / VEC;
    float xv[kAcc][VEC];
    if (full && a.x != nullptr) {                                   // the weights of a full tile are requested first
#pragma unroll
        for (int i = 0; i < kAcc; ++i) load_vals<VEC>(static_cast<XT*>(a.x) + cbase + (i * kWave + lane) * VEC, xv[i]);
    }
    float acc[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) acc[c] = 0.0f;
    constexpr int UM = 4;                                           // workers whose plane dwords are in flight together
    for (int m0 = 0; m0 < a.M; m0 += UM) {
        uint32_t nz[UM], sg[UM];
#pragma unroll
        for (int k = 0; k < UM; ++k) {
            const bool on = have && m0 + k < a.M;
            nz[k] = on ? stream_load(nzp + (int64_t)(m0 + k) * row_dw) : 0u;
            sg[k] = on ? stream_load(sgp + (int64_t)(m0 + k) * row_dw) : 0u;
        }
#pragma unroll
        for (int k = 0; k < UM; ++k) {                              // workers in index order: the fp32 sum has a fixed order
            if (m0 + k >= a.M) continue;
            const float nm = a.norms[m0 + k];
            if ((__float_as_uint(nm) & 0x7f800000u) != 0x7f800000u) {               // finite (workgroup-uniform)
#pragma unroll
                for (int q4 = 0; q4 < 8; ++q4) {
                    const uint32_t idx = ((nz[k] >> (4 * q4)) & 15u) | (((sg[k] >> (4 * q4)) & 15u) << 4);
                    const h16x4 f = factor[idx];                   // widened exactly inside the mixed-precision fma
                    acc[4 * q4 + 0] = fmaf(nm, (float)f.x, acc[4 * q4 + 0]);
                    acc[4 * q4 + 1] = fmaf(nm, (float)f.y, acc[4 * q4 + 1]);
                    acc[4 * q4 + 2] = fmaf(nm, (float)f.z, acc[4 * q4 + 2]);
                    acc[4 * q4 + 3] = fmaf(nm, (float)f.w, acc[4 * q4 + 3]);
                }
            } else {
                // Inf or NaN norm: the addend is +norm, -norm or +0, selected by all-ones / all-zeros masks from
                // one-bit signed bit-field extracts
                const uint32_t plus = __float_as_uint(nm), minus = plus ^ 0x80000000u;
                const uint32_t P = nz[k] & sg[k], N = nz[k] & ~sg[k];
#pragma unroll
                for (int c = 0; c < 32; ++c) {
                    const uint32_t mp = (uint32_t)__builtin_amdgcn_sbfe((int)P, c, 1);
                    const uint32_t mn = (uint32_t)__builtin_amdgcn_sbfe((int)N, c, 1);
                    acc[c] += __uint_as_float((mp & plus) | (mn & minus));
                }
            }
        }
    }
    float* st = stage[wave];
#pragma unroll
    for (int c = 0; c < 32; ++c) st[lane * kPad + c] = acc[c] * a.inv_m;       // coordinate 32 l + c of the tile
    // the wave's own LDS writes are complete before its reads (same wave: only the counter wait is needed)
    __builtin_amdgcn_s_waitcnt(0xc07f);                                          // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();

    if (full) {
#pragma unroll
        for (int i = 0; i < kAcc; ++i) {
            const int off = (i * kWave + lane) * VEC;
            float av[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) av[c] = st[((off + c) >> 5) * kPad + ((off + c) & 31)];
            if (a.avg_out != nullptr) store_vals<VEC>(a.avg_out + cbase + off, av);
            if (a.x != nullptr) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) xv[i][c] = fmaf(-a.lr, av[c], xv[i][c]);
                store_vals<VEC>(static_cast<XT*>(a.x) + cbase + off, xv[i]);
            }
        }
        return;
    }
    for (int i = 0; i < kAcc; ++i) {                                             // the ragged last tile
        const int off = (i * kWave + lane) * VEC;
        const int64_t r = left - off;
        const int n = r >= VEC ? VEC : (r > 0 ? (int)r : 0);
        if (n == 0) continue;
        float av[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) av[c] = st[((off + c) >> 5) * kPad + ((off + c) & 31)];
        if (a.avg_out != nullptr) store_vals_guarded<float, VEC>(a.avg_out + cbase + off, n, av);
        if (a.x != nullptr) {
            XT* xp = static_cast<XT*>(a.x) + cbase + off;
            float xg[VEC];
            load_vals_guarded<XT, VEC>(xp, n, xg);
#pragma unroll
            for (int c = 0; c < VEC; ++c) xg[c] = fmaf(-a.lr, av[c], xg[c]);
            store_vals_guarded<XT, VEC>(xp, n, xg);
        }
    }
}

static inline bool aligned_to(const void* p, uintptr_t k) { return reinterpret_cast<uintptr_t>(p) % k == 0; }

// ---- scratch space inside the library, for callers that cannot allocate ----------------------------------------
// The partial results of ssv_qsgd_norms_static live in this array instead of a caller's workspace: room for
// kStaticMaxRows rows of kNormParts doubles (512 KiB).  Every GPU the library runs on holds its own copy at its
// own address for the life of the process.  In host code the name `scratch` is only a handle for
// hipGetSymbolAddress; kernels get the device address that call returns.
constexpr int kStaticMaxRows = 256;
static __device__ __align__(256) double scratch[(size_t)kStaticMaxRows * kNormParts];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.  nullptr on failure.
static double* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = static_cast<double*>(p);
    }
    return g_scratch_ptr[dev];
}

template <typename GT, int VEC>
static hipError_t launch_norms(const NormArgs& a, hipStream_t s) {
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    if (a.kind == SSV_QSGD_L2) {
        hipLaunchKernelGGL((qsgd_norm_partial_kernel<GT, VEC, true>), dim3(kNormParts, a.M), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL((qsgd_norm_finish_kernel<true>), dim3(a.M), dim3(kBlock), 0, s, a);
    } else {
        hipLaunchKernelGGL((qsgd_norm_partial_kernel<GT, VEC, false>), dim3(kNormParts, a.M), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL((qsgd_norm_finish_kernel<false>), dim3(a.M), dim3(kBlock), 0, s, a);
    }
    return hipGetLastError();
}

template <typename GT, int VEC>
static hipError_t launch_quantize(const QuantArgs& a, int M, hipStream_t s) {
    constexpr int64_t kTile = (int64_t)kWave * VEC;
    constexpr int64_t kBlockTiles = kWavesPerBlock * kQuantSub;
    const int64_t ntiles = (a.d + kTile - 1) / kTile;
    const int64_t nfull = a.d / (kTile * kBlockTiles);
    const int64_t grid = (ntiles + kBlockTiles - 1) / kBlockTiles;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();
    hipLaunchKernelGGL((qsgd_quantize_kernel<GT, VEC>), dim3((unsigned)grid, M), dim3(kBlock), 0, s, a, nfull, ntiles);
    return hipGetLastError();
}

template <typename XT, int VEC>
static hipError_t launch_aggregate(const AggArgs& a, hipStream_t s) {
    const int64_t ntiles = (a.d + kWave * 32 - 1) / (kWave * 32);
    const int64_t grid = (ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();
    hipLaunchKernelGGL((qsgd_aggregate_kernel<XT, VEC>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, ntiles);
    return hipGetLastError();
}

}  // namespace ssv

using namespace ssv;

extern "C" {

size_t ssv_qsgd_workspace_bytes(int M) {
    if (M < 1 || M > SSV_MAX_WORKERS) return 0;
    return (size_t)M * kNormParts * sizeof(double);
}

int ssv_qsgd_norms(const void* g, int g_dt, int M, int64_t d, int64_t g_row_stride, int kind, float* norms,
                   void* workspace, size_t workspace_bytes, void* stream) {
    if (g == nullptr || norms == nullptr || workspace == nullptr) return SSV_ERR_NULL;
    if (g_dt != SSV_F32 && g_dt != SSV_BF16) return SSV_ERR_DTYPE;
    if (M < 1 || M > SSV_MAX_WORKERS || d < 1 || d > SSV_MAX_COORDS || g_row_stride < d) return SSV_ERR_SHAPE;
    if (kind != SSV_QSGD_L2 && kind != SSV_QSGD_MAX) return SSV_ERR_PARAM;
    if (workspace_bytes < ssv_qsgd_workspace_bytes(M)) return SSV_ERR_SHAPE;
    const uintptr_t es = g_dt == SSV_F32 ? 4 : 2;
    if (!aligned_to(g, es) || !aligned_to(norms, 4) || !aligned_to(workspace, 8)) return SSV_ERR_ALIGN;
    NormArgs a = {g, static_cast<double*>(workspace), norms, d, g_row_stride, M, kind};
    const bool vec = aligned_to(g, 4 * es) && (M == 1 || g_row_stride % 4 == 0);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (g_dt == SSV_F32) e = vec ? launch_norms<float, 4>(a, s) : launch_norms<float, 1>(a, s);
    else e = vec ? launch_norms<bf16, 4>(a, s) : launch_norms<bf16, 1>(a, s);
    return e == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}

int ssv_qsgd_norms_static(const void* g, int g_dt, int M, int64_t d, int64_t g_row_stride, int kind, float* norms,
                          void* stream) {
    if (M > kStaticMaxRows) return SSV_ERR_SHAPE;          // the built-in scratch space holds 256 rows' partial results
    if (g == nullptr || norms == nullptr) return SSV_ERR_NULL;
    double* ws = scratch_on_current_device();
    if (ws == nullptr) return SSV_ERR_HIP;
    // Same validation and the same kernels as ssv_qsgd_norms.  Nothing needs clearing: every workgroup of the first
    // kernel writes its partial result before the finishing kernel reads it, whatever the array held before.
    return ssv_qsgd_norms(g, g_dt, M, d, g_row_stride, kind, norms, ws, sizeof(double) * (size_t)kStaticMaxRows * kNormParts,
                          stream);
}

int ssv_qsgd_quantize(const void* g, int g_dt, const float* u, const float* norms, int M, int64_t d,
                      int64_t g_row_stride, int64_t u_row_stride, uint64_t* nonzero, uint64_t* sign,
                      int64_t row_stride_words, void* stream) {
    if (g == nullptr || u == nullptr || norms == nullptr || nonzero == nullptr || sign == nullptr) return SSV_ERR_NULL;
    if (g_dt != SSV_F32 && g_dt != SSV_BF16) return SSV_ERR_DTYPE;
    const int64_t W = (d + 63) / 64;
    if (M < 1 || M > SSV_MAX_WORKERS || d < 1 || d > SSV_MAX_COORDS || g_row_stride < d || u_row_stride < d ||
        row_stride_words < W)
        return SSV_ERR_SHAPE;
    const uintptr_t es = g_dt == SSV_F32 ? 4 : 2;
    if (!aligned_to(g, es) || !aligned_to(u, 4) || !aligned_to(norms, 4) || !aligned_to(nonzero, 8) || !aligned_to(sign, 8))
        return SSV_ERR_ALIGN;
    QuantArgs a = {g, u, norms, nonzero, sign, d, g_row_stride, u_row_stride, row_stride_words, W};
    const bool vec = aligned_to(g, 4 * es) && aligned_to(u, 16) && (M == 1 || (g_row_stride % 4 == 0 && u_row_stride % 4 == 0));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (g_dt == SSV_F32) e = vec ? launch_quantize<float, 4>(a, M, s) : launch_quantize<float, 1>(a, M, s);
    else e = vec ? launch_quantize<bf16, 4>(a, M, s) : launch_quantize<bf16, 1>(a, M, s);
    return e == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}

int ssv_qsgd_aggregate_apply(const uint64_t* nonzero, const uint64_t* sign, const float* norms, int M, int64_t d,
                             int64_t row_stride_words, float* avg_out, void* x, int x_dt, float lr, void* stream) {
    if (nonzero == nullptr || sign == nullptr || norms == nullptr) return SSV_ERR_NULL;
    if (avg_out == nullptr && x == nullptr) return SSV_ERR_NULL;
    if (x != nullptr && x_dt != SSV_F32 && x_dt != SSV_BF16) return SSV_ERR_DTYPE;
    if (M < 1 || M > SSV_MAX_WORKERS || d < 1 || d > SSV_MAX_COORDS || row_stride_words < (d + 63) / 64) return SSV_ERR_SHAPE;
    if (x != nullptr && !std::isfinite(lr)) return SSV_ERR_PARAM;
    const uintptr_t xes = x_dt == SSV_F32 ? 4 : 2;
    if (!aligned_to(nonzero, 8) || !aligned_to(sign, 8) || !aligned_to(norms, 4) || !aligned_to(avg_out, 4)) return SSV_ERR_ALIGN;
    if (x != nullptr && !aligned_to(x, xes)) return SSV_ERR_ALIGN;
    AggArgs a = {nonzero, sign, norms, avg_out, x, d, row_stride_words, M, 1.0f / (float)M, lr};
    const bool vec = aligned_to(avg_out, 16) && (x == nullptr || aligned_to(x, 4 * xes));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (x == nullptr || x_dt == SSV_F32) e = vec ? launch_aggregate<float, 4>(a, s) : launch_aggregate<float, 1>(a, s);
    else e = vec ? launch_aggregate<bf16, 4>(a, s) : launch_aggregate<bf16, 1>(a, s);
    return e == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}

}  // extern "C"
