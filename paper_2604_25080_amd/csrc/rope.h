// The RoPE rotation of one (x[j], x[j + head_dim/2]) pair, spelled out operation by operation so
// that every kernel that rotates produces the same bits: two products rounded on their own, two
// fused multiply-adds.
#pragma once
#include <hip/hip_runtime.h>

namespace cf {

__device__ __forceinline__ void rope_rotate(float x1, float x2, float2 cos_sin, float& y1, float& y2) {
    y1 = __builtin_fmaf(x1, cos_sin.x, -(x2 * cos_sin.y));
    y2 = __builtin_fmaf(x2, cos_sin.x, x1 * cos_sin.y);
}

}  // namespace cf
