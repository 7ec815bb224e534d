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

int ssv_signum_step_multi(const void* plan_host, const void* plan_device, float beta, float lr, float weight_decay,
                          void* stream) {
    if (plan_host == nullptr || plan_device == nullptr) return SSV_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(plan_host) % 8 != 0 || reinterpret_cast<uintptr_t>(plan_device) % 8 != 0)
        return SSV_ERR_ALIGN;
    PlanHeader h;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != kPlanMagic || h.T < 1 || h.M < 1 || h.M > SSV_MAX_WORKERS || h.nunits < 1 ||
        h.nunits > 0x7fffffffLL || h.bytes < (int64_t)sizeof(PlanHeader))
        return SSV_ERR_SHAPE;
    if (!(beta >= 0.0f && beta < 1.0f)) return SSV_ERR_PARAM;
    if (!h.has_v && beta != 0.0f) return SSV_ERR_PARAM;
    if (!std::isfinite(lr) || !std::isfinite(weight_decay)) return SSV_ERR_PARAM;
    const unsigned char* base = static_cast<const unsigned char*>(plan_device);
    MultiArgs ma;
    ma.first_unit = reinterpret_cast<const int64_t*>(base + h.off_first_unit);
    ma.n = reinterpret_cast<const int64_t*>(base + h.off_n);
    ma.x = reinterpret_cast<void* const*>(base + h.off_x);
    ma.g = reinterpret_cast<const void* const*>(base + h.off_g);
    ma.v = reinterpret_cast<float* const*>(base + h.off_v);
    ma.unit_tensor = reinterpret_cast<const int32_t*>(base + h.off_unit_tensor);
    ma.aligned = base + h.off_aligned;
    ma.M = (int)h.M; ma.T = ((int)h.M + 1) / 2;
    ma.beta = beta; ma.omb = 1.0f - beta; ma.lr = lr; ma.wd = weight_decay;
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

}  // extern "C"
