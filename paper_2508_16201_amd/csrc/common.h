// Shared device/host helpers for the gfx950 kernels (wave64, MFMA 16x16x32 bf16).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "specvlm.h"

namespace specvlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kNumXcd = 8;          // MI355X: 8 accelerator dies, each with its own L2
constexpr int kNumCu = 256;

// D = A(16x32 bf16) * B(32x16 bf16) + C.  Per lane (r = lane % 16, c = lane / 16):
//   A holds row r,    contraction indices 8c..8c+7
//   B holds column r, contraction indices 8c..8c+7
//   C/D hold column r, rows 4c..4c+3
__device__ __forceinline__ floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Workgroups are dealt to the XCDs round-robin by linear id.  Map the hardware
// id to a logical id so that consecutive logical ids share an XCD (and its L2).
// `padded` is the launch size, a multiple of kNumXcd; ids >= the real count exit.
__device__ __forceinline__ int xcd_logical_id(int hw_id, int padded)
{
    const int per_xcd = padded / kNumXcd;
    return (hw_id % kNumXcd) * per_xcd + hw_id / kNumXcd;
}

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? SPECVLM_OK : SPECVLM_ELAUNCH;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

}  // namespace specvlm
