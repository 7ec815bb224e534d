// Multi-tensor form of the fused Signum step: the parameters of a model are T separate tensors, and every
// worker's gradient (and momentum) of a tensor is an allocation of its own.  One launch covers all of them:
// the index space is the concatenation of the tensors cut into units of 4096 coordinates, the last unit of
// each tensor being ragged, and a workgroup looks up the tensor of its unit in a table that the caller
// built once (the "plan") and keeps in device memory.  Inside a unit the work is exactly the flat kernel's
// (step_tiles.h), with worker rows addressed through the table's per-worker pointers.
//
// This is the tensor fusion of Section 4 of the paper (small tensors fused to save compression and
// communication cost) done by indexing instead of by copying gradients into a flat buffer.
#include <cmath>
#include <cstring>

#include "../../include/signvote.h"
#include "step_tiles.h"
#include "vote_tiles.h"

namespace ssv {

constexpr int64_t kUnit = (int64_t)kWave * 4 * kWavesPerBlock * kStepSub;     // 4096 coordinates
constexpr uint64_t kPlanMagic = 0x314e414c50565353ull;                        // "SSVPLAN1"

// Header of the plan; the arrays follow at the byte offsets it names.  Only offsets, no addresses of the
// plan itself, so the same bytes are valid on the host and on the device.
struct PlanHeader {
    uint64_t magic;
    int64_t bytes;
    int64_t T, M, nunits, total_n;
    int64_t g_dt, x_dt, has_v;
    int64_t off_first_unit;   // int64 [T + 1]  units before tensor t
    int64_t off_n;            // int64 [T]      elements of tensor t
    int64_t off_x;            // void* [T]      weights
    int64_t off_g;            // void* [T * M]  gradients, tensor-major
    int64_t off_v;            // float* [T * M] momenta, tensor-major (unused without momentum)
    int64_t off_unit_tensor;  // int32 [nunits] tensor of every unit
    int64_t off_aligned;      // uint8 [T]      1 = every pointer of the tensor allows 4-element vector accesses
};

static inline int64_t round8(int64_t b) { return (b + 7) & ~int64_t(7); }

static bool plan_layout(int T, int M, const int64_t* n, PlanHeader& h) {
    if (T < 1 || M < 1 || M > SSV_MAX_WORKERS || n == nullptr) return false;
    int64_t units = 0, total = 0;
    for (int t = 0; t < T; ++t) {
        if (n[t] < 1 || n[t] > SSV_MAX_COORDS) return false;
        units += (n[t] + kUnit - 1) / kUnit;
        total += n[t];
        if (total > SSV_MAX_COORDS) return false;
    }
    if (units > 0x7fffffffLL) return false;
    h = PlanHeader{};
    h.magic = kPlanMagic;
    h.T = T; h.M = M; h.nunits = units; h.total_n = total;
    int64_t off = round8((int64_t)sizeof(PlanHeader));
    h.off_first_unit = off; off += 8 * (int64_t)(T + 1);
    h.off_n = off; off += 8 * (int64_t)T;
    h.off_x = off; off += 8 * (int64_t)T;
    h.off_g = off; off += 8 * (int64_t)T * M;
    h.off_v = off; off += 8 * (int64_t)T * M;
    h.off_unit_tensor = off; off += round8(4 * units);
    h.off_aligned = off; off += round8(T);
    h.bytes = off;
    return true;
}

struct MultiArgs {
    const int64_t* first_unit;
    const int64_t* n;
    void* const* x;
    const void* const* g;
    float* const* v;
    const int32_t* unit_tensor;
    const uint8_t* aligned;
    int M, T;
    float beta, omb, lr, wd;
    // two-kernel form only: the packed signs of all workers, M rows of 64 words per unit (a unit's 4096 sign bits)
    uint64_t* signs;
    int64_t signs_stride;     // words per row = 64 * nunits
    uint32_t init;            // preload 2^k - T of the bit-sliced vote counter
};

// The last, partial unit of a tensor, and every unit of a tensor with a pointer that does not allow vector
// accesses: bounds-checked tiles, one at a time.  Kept out of line so that its registers do not count against
// the hot path of the kernel, which sits exactly at the register budget of five waves per SIMD.
// Takes the tensor's description as plain values (a reference to a StepArgs would force that struct, and with it
// the hot path's copy, into memory).
template <typename GT, typename XT, bool MOM>
__device__ __attribute__((noinline)) void ragged_or_unaligned_unit(const void* g, float* v, void* x, int64_t n, int M,
                                                                   int T, float beta, float omb, float lr, float wd,
                                                                   int64_t u, bool aligned, int wave, int lane) {
    StepArgs a;
    a.g = g; a.v = v; a.x = x; a.vote_out = nullptr; a.signs_out = nullptr;
    a.d = n; a.M = M; a.T = T; a.beta = beta; a.omb = omb; a.lr = lr; a.wd = wd; a.has_flip = 0;
    if (aligned) {
        constexpr int64_t kTileCoords = (int64_t)kWave * 4;
        for (int s = 0; s < kStepSub; ++s) {
            const int64_t tile = u * (kWavesPerBlock * kStepSub) + wave + s * kWavesPerBlock;
            if (tile * kTileCoords < a.d) step_tiles<GT, XT, 4, 1, MOM, true, false, true, false, TableRows>(a, tile, lane);
        }
    } else {
        // one coordinate per lane: the unit's 4096 coordinates are 64 tiles of 64
        constexpr int kTilesPerWave = (int)(kUnit / kWave / kWavesPerBlock);
        for (int s = 0; s < kTilesPerWave; ++s) {
            const int64_t tile = u * (kUnit / kWave) + wave + (int64_t)s * kWavesPerBlock;
            if (tile * kWave < a.d) step_tiles<GT, XT, 1, 1, MOM, true, false, true, false, TableRows>(a, tile, lane);
        }
    }
}

template <typename GT, typename XT, bool MOM, bool SERIAL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(5, 5))) void step_multi_kernel(MultiArgs ma) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);      // tell the compiler it is wave-uniform
    const int64_t unit = blockIdx.x;
    const int t = ma.unit_tensor[unit];                       // workgroup-uniform: scalar loads
    const int64_t u = unit - ma.first_unit[t];                // unit inside its tensor

    StepArgs a;                                               // only the fields the lean form reads
    a.g = ma.g + (int64_t)t * ma.M;
    a.v = MOM ? reinterpret_cast<float*>(const_cast<float**>(ma.v + (int64_t)t * ma.M)) : nullptr;
    a.x = ma.x[t];
    a.vote_out = nullptr; a.signs_out = nullptr;
    a.d = ma.n[t];
    a.M = ma.M; a.T = ma.T;
    a.beta = ma.beta; a.omb = ma.omb; a.lr = ma.lr; a.wd = ma.wd;
    a.has_flip = 0;

    if (ma.aligned[t] && (u + 1) * kUnit <= a.d) {
        // the common case, a whole unit of an aligned tensor: exactly the flat kernel's inner body
        step_tiles<GT, XT, 4, kStepSub, MOM, true, false, false, SERIAL, TableRows>(
            a, u * (kWavesPerBlock * kStepSub) + wave, lane);
    } else {
        ragged_or_unaligned_unit<GT, XT, MOM>(a.g, a.v, a.x, a.d, a.M, a.T, a.beta, a.omb, a.lr, a.wd, u,
                                              ma.aligned[t] != 0, wave, lane);
    }
}

// ---- two-kernel form (ssv_signum_step_multi_ws) ---------------------------------------------------------------
// As for the flat vector (step_kernels.hip, pack_rows_kernel): momentum + sign + pack one worker after the other on
// a grid (quarter units, M), the packed signs going to the caller's workspace, then vote + update on the packed
// rows.  In the workspace every unit owns 64 words of each worker's row, so a tensor's words start at word
// 64 * first_unit[t]; words past a tensor's end inside its last unit are never written and never read.
template <typename GT, bool MOM, bool SERIAL>
__global__ __launch_bounds__(kBlock) void pack_multi_kernel(MultiArgs ma) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);      // tell the compiler it is wave-uniform
    const int m = blockIdx.y;
    const int64_t unit = blockIdx.x >> 2;
    const int quarter = blockIdx.x & 3;                       // 1024 coordinates: one tile of 256 per wave
    const int t = ma.unit_tensor[unit];                       // workgroup-uniform: scalar loads
    const int64_t first = ma.first_unit[t];
    const int64_t n = ma.n[t];

    StepArgs a;                                               // only the fields worker_group reads
    a.signs_out = ma.signs + (int64_t)m * ma.signs_stride + 64 * first;
    a.signs_stride = 0;                                       // the row is already selected
    a.W = (n + 63) / 64;
    a.beta = ma.beta; a.omb = ma.omb;
    a.has_flip = 0;
    RowStarts<GT, 1> row;
    row.g[0] = reinterpret_cast<const GT*>(uniform_table_entry(ma.g, (int64_t)t * ma.M + m));
    row.v[0] = MOM ? reinterpret_cast<float*>(uniform_table_entry(ma.v, (int64_t)t * ma.M + m)) : nullptr;
    const int64_t c0 = (unit - first) * kUnit + quarter * (kUnit / 4);     // first coordinate of the workgroup, in the tensor
    if (c0 >= n) return;                                                   // workgroup-uniform
    if (ma.aligned[t]) {
        const int64_t tile = c0 / 256 + wave;
        const uint32_t jl = (uint32_t)lane * 4;
        uint32_t unused_count[1][2] = {};
        if ((tile + 1) * 256 <= n) {
            int nvalid[1] = {4};
            worker_group<GT, 4, 1, MOM, true, false, SERIAL, 1>(a, row, 0, tile * 256, jl, nvalid, lane, tile, unused_count);
        } else if (tile * 256 < n) {
            const int64_t left = n - (tile * 256 + jl);
            int nvalid[1] = {left >= 4 ? 4 : (left > 0 ? (int)left : 0)};
            worker_group<GT, 4, 1, MOM, true, true, false, 1>(a, row, 0, tile * 256, jl, nvalid, lane, tile, unused_count);
        }
    } else {
        // one coordinate per lane: the workgroup's 1024 coordinates are 16 tiles of 64, wave w taking w, w+4, ..
        for (int k = 0; k < 4; ++k) {
            const int64_t tile = c0 / 64 + wave + 4 * k;
            if (tile * 64 >= n) break;                                     // wave-uniform
            const int64_t left = n - (tile * 64 + lane);
            int nvalid[1] = {left > 0 ? 1 : 0};
            uint32_t unused_count[1][1] = {};
            worker_group<GT, 1, 1, MOM, true, true, false, 1>(a, row, 0, tile * 64, (uint32_t)lane, nvalid, lane, tile,
                                                              unused_count);
        }
    }
}

// One wave per half unit (2048 coordinates, 32 words of every workspace row).
template <int NPL, typename XT, int XV>
__global__ __launch_bounds__(kBlock) void vote_apply_multi_kernel(MultiArgs ma, int64_t ntiles) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tile >= ntiles) return;                               // wave-uniform
    const int64_t unit = tile >> 1;
    const int t = ma.unit_tensor[unit];
    const int64_t n = ma.n[t];
    const int64_t c0 = (unit - ma.first_unit[t]) * kUnit + (tile & 1) * (kUnit / 2);   // in the tensor
    if (c0 >= n) return;                                      // wave-uniform: the half unit lies past the tensor's end
    const int64_t rem = n - (c0 + 32 * lane);                 // coordinates from this lane's first bit on
    XT* xt = static_cast<XT*>(ma.x[t]) + c0;
    const uint32_t* p = reinterpret_cast<const uint32_t*>(ma.signs) + tile * kWave + lane;
    if (ma.aligned[t])
        vote_apply_tile<NPL, XT, XV>(p, 2 * ma.signs_stride, ma.M, ma.init, rem > 0, rem, xt, n - c0, nullptr, ma.lr, ma.wd, lane);
    else
        vote_apply_tile<NPL, XT, 1>(p, 2 * ma.signs_stride, ma.M, ma.init, rem > 0, rem, xt, n - c0, nullptr, ma.lr, ma.wd, lane);
}

template <typename GT, bool MOM>
static hipError_t launch_pack_multi(const MultiArgs& ma, int64_t nunits, hipStream_t s) {
    if (4 * nunits > 0x7fffffffLL || ma.M > 65535) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    const dim3 grid((unsigned)(4 * nunits), (unsigned)ma.M);
    if (MOM && tuning().step_serial) hipLaunchKernelGGL((pack_multi_kernel<GT, MOM, MOM>), grid, dim3(kBlock), 0, s, ma);
    else hipLaunchKernelGGL((pack_multi_kernel<GT, MOM, false>), grid, dim3(kBlock), 0, s, ma);
    return hipGetLastError();
}

template <int NPL>
static hipError_t launch_vote_apply_multi(const MultiArgs& ma, int x_dt, int64_t nunits, hipStream_t s) {
    const int64_t ntiles = 2 * nunits;
    if (ntiles > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    (void)hipGetLastError();
    // single-wave workgroups: the workspace rows start on cache-line boundaries (see launch_vote_apply_one)
    if (x_dt == SSV_F32) hipLaunchKernelGGL((vote_apply_multi_kernel<NPL, float, 4>), dim3((unsigned)ntiles), dim3(kWave), 0, s, ma, ntiles);
    else hipLaunchKernelGGL((vote_apply_multi_kernel<NPL, bf16, 4>), dim3((unsigned)ntiles), dim3(kWave), 0, s, ma, ntiles);
    return hipGetLastError();
}

template <typename GT, typename XT, bool MOM>
static hipError_t launch_multi(const MultiArgs& ma, int64_t nunits, hipStream_t s) {
    (void)hipGetLastError();                 // a stale error of an earlier, unrelated call is not this launch's
    if (MOM && tuning().step_serial)
        hipLaunchKernelGGL((step_multi_kernel<GT, XT, MOM, MOM>), dim3((unsigned)nunits), dim3(kBlock), 0, s, ma);
    else
        hipLaunchKernelGGL((step_multi_kernel<GT, XT, MOM, false>), dim3((unsigned)nunits), dim3(kBlock), 0, s, ma);
    return hipGetLastError();
}

template <typename GT, typename XT>
static hipError_t launch_multi_mom(const MultiArgs& ma, bool mom, int64_t nunits, hipStream_t s) {
    return mom ? launch_multi<GT, XT, true>(ma, nunits, s) : launch_multi<GT, XT, false>(ma, nunits, s);
}

}  // namespace ssv

using namespace ssv;

extern "C" {

size_t ssv_multi_plan_bytes(int T, int M, const int64_t* n) {
    PlanHeader h;
    return plan_layout(T, M, n, h) ? (size_t)h.bytes : 0;
}

int ssv_multi_plan_fill(void* plan_host, size_t plan_bytes, int T, int M, const int64_t* n, void* const* x, int x_dt,
                        const void* const* g, int g_dt, float* const* v) {
    if (plan_host == nullptr || n == nullptr || x == nullptr || g == nullptr) return SSV_ERR_NULL;
    if ((g_dt != SSV_F32 && g_dt != SSV_BF16) || (x_dt != SSV_F32 && x_dt != SSV_BF16)) return SSV_ERR_DTYPE;
    PlanHeader h;
    if (!plan_layout(T, M, n, h)) return SSV_ERR_SHAPE;
    if (plan_bytes < (size_t)h.bytes) return SSV_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(plan_host) % 8 != 0) return SSV_ERR_ALIGN;
    const uintptr_t ges = g_dt == SSV_F32 ? 4 : 2, xes = x_dt == SSV_F32 ? 4 : 2;
    for (int t = 0; t < T; ++t) {
        if (x[t] == nullptr) return SSV_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(x[t]) % xes != 0) return SSV_ERR_ALIGN;
        for (int m = 0; m < M; ++m) {
            const void* gp = g[(int64_t)t * M + m];
            if (gp == nullptr || (v != nullptr && v[(int64_t)t * M + m] == nullptr)) return SSV_ERR_NULL;
            if (reinterpret_cast<uintptr_t>(gp) % ges != 0) return SSV_ERR_ALIGN;
            if (v != nullptr && reinterpret_cast<uintptr_t>(v[(int64_t)t * M + m]) % 4 != 0) return SSV_ERR_ALIGN;
        }
    }
    h.g_dt = g_dt; h.x_dt = x_dt; h.has_v = v != nullptr;
    unsigned char* base = static_cast<unsigned char*>(plan_host);
    std::memset(base, 0, (size_t)h.bytes);
    std::memcpy(base, &h, sizeof(h));
    int64_t* first_unit = reinterpret_cast<int64_t*>(base + h.off_first_unit);
    int64_t* nn = reinterpret_cast<int64_t*>(base + h.off_n);
    void** xx = reinterpret_cast<void**>(base + h.off_x);
    const void** gg = reinterpret_cast<const void**>(base + h.off_g);
    float** vv = reinterpret_cast<float**>(base + h.off_v);
    int32_t* unit_tensor = reinterpret_cast<int32_t*>(base + h.off_unit_tensor);
    uint8_t* aligned = base + h.off_aligned;
    int64_t units = 0;
    for (int t = 0; t < T; ++t) {
        first_unit[t] = units;
        nn[t] = n[t];
        xx[t] = x[t];
        // 4 elements per lane: 16-byte pieces of fp32, 8-byte pieces of bf16
        bool ok = reinterpret_cast<uintptr_t>(x[t]) % (4 * xes) == 0;
        for (int m = 0; m < M; ++m) {
            gg[(int64_t)t * M + m] = g[(int64_t)t * M + m];
            ok = ok && reinterpret_cast<uintptr_t>(g[(int64_t)t * M + m]) % (4 * ges) == 0;
            if (v != nullptr) {
                vv[(int64_t)t * M + m] = v[(int64_t)t * M + m];
                ok = ok && reinterpret_cast<uintptr_t>(v[(int64_t)t * M + m]) % 16 == 0;
            }
        }
        aligned[t] = ok ? 1 : 0;
        const int64_t ut = (n[t] + kUnit - 1) / kUnit;
        for (int64_t k = 0; k < ut; ++k) unit_tensor[units + k] = t;
        units += ut;
    }
    first_unit[T] = units;
    return SSV_OK;
}

// Validates the plan header and the step parameters, fills the kernel arguments.  Returns SSV_OK or an error code.
static int multi_args(const void* plan_host, const void* plan_device, float beta, float lr, float weight_decay,
                      PlanHeader& h, MultiArgs& ma) {
    if (plan_host == nullptr || plan_device == nullptr) return SSV_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan_host) % 8 != 0 || reinterpret_cast<uintptr_t>(plan_device) % 8 != 0)
        return SSV_ERR_ALIGN;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != kPlanMagic || h.T < 1 || h.M < 1 || h.M > SSV_MAX_WORKERS || h.nunits < 1 ||
        h.nunits > 0x7fffffffLL || h.bytes < (int64_t)sizeof(PlanHeader))
        return SSV_ERR_SHAPE;
    if (!(beta >= 0.0f && beta < 1.0f)) return SSV_ERR_PARAM;
    if (!h.has_v && beta != 0.0f) return SSV_ERR_PARAM;
    if (!std::isfinite(lr) || !std::isfinite(weight_decay)) return SSV_ERR_PARAM;
    const unsigned char* base = static_cast<const unsigned char*>(plan_device);
    ma = MultiArgs{};
    ma.first_unit = reinterpret_cast<const int64_t*>(base + h.off_first_unit);
    ma.n = reinterpret_cast<const int64_t*>(base + h.off_n);
    ma.x = reinterpret_cast<void* const*>(base + h.off_x);
    ma.g = reinterpret_cast<const void* const*>(base + h.off_g);
    ma.v = reinterpret_cast<float* const*>(base + h.off_v);
    ma.unit_tensor = reinterpret_cast<const int32_t*>(base + h.off_unit_tensor);
    ma.aligned = base + h.off_aligned;
    ma.M = (int)h.M; ma.T = ((int)h.M + 1) / 2;
    ma.beta = beta; ma.omb = 1.0f - beta; ma.lr = lr; ma.wd = weight_decay;
    return SSV_OK;
}

int ssv_signum_step_multi(const void* plan_host, const void* plan_device, float beta, float lr, float weight_decay,
                          void* stream) {
    PlanHeader h;
    MultiArgs ma;
    if (int rc = multi_args(plan_host, plan_device, beta, lr, weight_decay, h, ma)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mom = h.has_v != 0;
    hipError_t e;
    if (h.g_dt == SSV_F32)
        e = h.x_dt == SSV_F32 ? launch_multi_mom<float, float>(ma, mom, h.nunits, s)
                              : launch_multi_mom<float, bf16>(ma, mom, h.nunits, s);
    else
        e = h.x_dt == SSV_F32 ? launch_multi_mom<bf16, float>(ma, mom, h.nunits, s)
                              : launch_multi_mom<bf16, bf16>(ma, mom, h.nunits, s);
    return e == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}

size_t ssv_multi_workspace_bytes(const void* plan_host) {
    if (plan_host == nullptr || reinterpret_cast<uintptr_t>(plan_host) % 8 != 0) return 0;
    PlanHeader h;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != kPlanMagic || h.M < 1 || h.M > SSV_MAX_WORKERS || h.nunits < 1 || h.nunits > 0x7fffffffLL) return 0;
    return (size_t)h.M * (size_t)h.nunits * 64 * sizeof(uint64_t);
}

int ssv_signum_step_multi_ws(const void* plan_host, const void* plan_device, void* workspace, size_t workspace_bytes,
                             float beta, float lr, float weight_decay, void* stream) {
    PlanHeader h;
    MultiArgs ma;
    if (int rc = multi_args(plan_host, plan_device, beta, lr, weight_decay, h, ma)) return rc;
    if (workspace == nullptr) return SSV_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return SSV_ERR_ALIGN;
    if (workspace_bytes < ssv_multi_workspace_bytes(plan_host)) return SSV_ERR_SHAPE;
    ma.signs = static_cast<uint64_t*>(workspace);
    ma.signs_stride = 64 * h.nunits;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mom = h.has_v != 0;
    hipError_t e;
    if (h.g_dt == SSV_F32) e = mom ? launch_pack_multi<float, true>(ma, h.nunits, s) : launch_pack_multi<float, false>(ma, h.nunits, s);
    else e = mom ? launch_pack_multi<bf16, true>(ma, h.nunits, s) : launch_pack_multi<bf16, false>(ma, h.nunits, s);
    if (e != hipSuccess) return SSV_ERR_HIP;
    const int T = (ma.M + 1) / 2;                              // vote threshold; counter planes as in launch_vote
    if (ma.M <= 15) { ma.init = (1u << 3) - T; e = launch_vote_apply_multi<4>(ma, (int)h.x_dt, h.nunits, s); }
    else if (ma.M <= 63) { ma.init = (1u << 5) - T; e = launch_vote_apply_multi<6>(ma, (int)h.x_dt, h.nunits, s); }
    else if (ma.M <= 255) { ma.init = (1u << 7) - T; e = launch_vote_apply_multi<8>(ma, (int)h.x_dt, h.nunits, s); }
    else { ma.init = (1u << 9) - T; e = launch_vote_apply_multi<10>(ma, (int)h.x_dt, h.nunits, s); }
    return e == hipSuccess ? SSV_OK : SSV_ERR_HIP;
}

}  // extern "C"
