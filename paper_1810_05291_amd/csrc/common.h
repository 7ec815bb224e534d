// Internal declarations shared by the HIP translation units of libsignvote (gfx950 only).
// Nothing here is part of the public C ABI (that is include/signvote.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssv {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kBlock = 256;          // threads per workgroup = 4 wavefronts
constexpr int kWavesPerBlock = kBlock / kWave;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct bf16 { uint16_t bits; };      // storage-only bf16

// One bit per worker: set = that worker transmits the negation of its signs.
struct FlipMask { uint32_t w[32]; };

// ---- number formats -------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h16) { return __uint_as_float(h16 << 16); }

// fp32 -> bf16, round to nearest even on the bit pattern; NaN keeps sign/payload top bits, quieted.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : rounded;
}

// ---- launch plumbing ---------------------------------------------------------------------------
struct StepArgs {
    const void* g;          // [M][g_stride] gradients (fp32 or bf16)
    float* v;               // [M][v_stride] momentum, or nullptr
    void* x;                // [d] weights, or nullptr (no update)
    uint64_t* vote_out;     // [W] or nullptr
    uint64_t* signs_out;    // [M][signs_stride] or nullptr
    int64_t d, g_stride, v_stride, signs_stride, W;
    int64_t ntiles;         // wave tiles of 64*VEC coordinates
    int M, T;               // workers, vote threshold (M+1)/2
    float beta, omb, lr, wd;
    int has_flip;
    FlipMask flip;
};

struct VoteArgs {
    const uint64_t* signs;  // [M][stride_words]
    uint64_t* vote_out;     // [W] or nullptr
    void* x;                // [d] or nullptr
    int64_t d, W, stride_words;
    int64_t ntiles;         // wave tiles of 64*PW dwords
    int M;
    uint32_t init;          // 2^k - T: preload of the bit-sliced counter
    float lr, wd;
};

struct ApplyArgs {
    void* x;
    const uint64_t* vote;
    int64_t d;
    float lr, wd;
};

// Each returns hipSuccess or the launch error.  dtypes: 0 = fp32, 1 = bf16.
hipError_t launch_step(const StepArgs& a, int g_dt, int x_dt, bool vector_ok, hipStream_t s);
hipError_t launch_vote(const VoteArgs& a, int x_dt, bool rows16, bool x_vector_ok, hipStream_t s);
hipError_t launch_apply(const ApplyArgs& a, int x_dt, bool x_vector_ok, hipStream_t s);

// Measurement switch, read once per process from the environment (documented in include/signvote.h).
struct Tuning {
    int step_serial;           // 1 (default) = one row load in flight per wave in the momentum forms of the step kernel
};
const Tuning& tuning();

}  // namespace ssv
