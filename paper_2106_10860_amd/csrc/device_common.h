// Device-side helpers shared by the kernels of libmaddness.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

// A lambda that must become part of its caller: as a call, what it captures by reference
// (kernel arguments, register arrays) would go through memory.
#define INLINE_LAMBDA __attribute__((always_inline))

namespace maddness {

// Make LDS writes of this wavefront visible to its other lanes.  The hardware
// executes the LDS operations of one wavefront in order; this only stops the
// compiler from moving accesses across the point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Element types of A (the values of maddness_dtype).  Every element is widened to
// the fp32 number of the same value before it is compared with a threshold:
// exact for binary16, bfloat16 (the upper half of an fp32) and unsigned bytes.
enum : int { kF32 = 0, kF16 = 1, kBF16 = 2, kU8 = 3 };

__host__ __device__ constexpr int elem_size(int dt) { return dt == kF32 ? 4 : (dt == kU8 ? 1 : 2); }

template <int DT>
__device__ __forceinline__ float widen_at(const void *base, int64_t idx)
{
    if constexpr (DT == kF32) return static_cast<const float *>(base)[idx];
    else if constexpr (DT == kF16) return (float)static_cast<const _Float16 *>(base)[idx];
    else if constexpr (DT == kBF16) return __uint_as_float((uint32_t) static_cast<const uint16_t *>(base)[idx] << 16);
    else return (float)static_cast<const uint8_t *>(base)[idx];
}

// the same with the type chosen at run time (wavefront-uniform)
__device__ __forceinline__ float widen_at(const void *base, int dt, int64_t idx)
{
    switch (dt) {
    case kF32: return widen_at<kF32>(base, idx);
    case kF16: return widen_at<kF16>(base, idx);
    case kBF16: return widen_at<kBF16>(base, idx);
    default: return widen_at<kU8>(base, idx);
    }
}

// The 15 thresholds of one tree held in registers; the node is chosen with
// selects instead of an indexed read.
struct Tree {
    int j0, j1, j2, j3;
    float t[15];
};

__device__ __forceinline__ void load_tree(Tree &tr, const int32_t *sd, const float *th, int D)
{
    tr.j0 = min(max(sd[0], 0), D - 1);
    tr.j1 = min(max(sd[1], 0), D - 1);
    tr.j2 = min(max(sd[2], 0), D - 1);
    tr.j3 = min(max(sd[3], 0), D - 1);
#pragma unroll
    for (int i = 0; i < 15; ++i) tr.t[i] = th[i];
}

__device__ __forceinline__ unsigned hash_regs(const Tree &tr, float x0, float x1, float x2, float x3)
{
    const bool b1 = x0 >= tr.t[0];
    const float v2 = b1 ? tr.t[2] : tr.t[1];
    const bool b2 = x1 >= v2;
    const float v3l = b2 ? tr.t[4] : tr.t[3];
    const float v3r = b2 ? tr.t[6] : tr.t[5];
    const float v3 = b1 ? v3r : v3l;
    const bool b3 = x2 >= v3;
    const float v4a = b3 ? tr.t[8] : tr.t[7];
    const float v4b = b3 ? tr.t[10] : tr.t[9];
    const float v4c = b3 ? tr.t[12] : tr.t[11];
    const float v4d = b3 ? tr.t[14] : tr.t[13];
    const float v4l = b2 ? v4b : v4a;
    const float v4r = b2 ? v4d : v4c;
    const float v4 = b1 ? v4r : v4l;
    const bool b4 = x3 >= v4;
    return (b1 ? 8u : 0u) | (b2 ? 4u : 0u) | (b3 ? 2u : 0u) | (b4 ? 1u : 0u);
}

}  // namespace maddness
