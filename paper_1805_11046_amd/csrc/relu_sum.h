// Optional last step of a layer-gradient convolution's epilogue (network plumbing, not from the paper): the
// gradient that leaves a residual block towards its input, res = act > 0 ? dx + other : 0, with dx the value the
// epilogue is about to store, other the gradient of the block's other branch (nullable: nothing added) and act the
// block's input, whose rectifier the gradient passes.  One fp32 addition, as q8t_relu_bwd_sum performs it, so the
// fused call and the two separate ones agree bit for bit.  act == NULL: nothing happens.
#pragma once
#include <hip/hip_runtime.h>

struct Q8tReluSum {
    const float *other;
    const float *act;
};

__device__ __forceinline__ float q8t_relu_sum1(const Q8tReluSum &f, size_t o, float v)
{
    if (f.act) {
        if (f.other) v = v + f.other[o];
        v = f.act[o] > 0.0f ? v : 0.0f;
    }
    return v;
}

__device__ __forceinline__ float2 q8t_relu_sum2(const Q8tReluSum &f, size_t o, float2 v)
{
    if (f.act) {
        if (f.other) {
            const float2 t = *reinterpret_cast<const float2 *>(f.other + o);
            v.x = v.x + t.x;
            v.y = v.y + t.y;
        }
        const float2 a = *reinterpret_cast<const float2 *>(f.act + o);
        v.x = a.x > 0.0f ? v.x : 0.0f;
        v.y = a.y > 0.0f ? v.y : 0.0f;
    }
    return v;
}

__device__ __forceinline__ float4 q8t_relu_sum4(const Q8tReluSum &f, size_t o, float4 v)
{
    if (f.act) {
        if (f.other) {
            const float4 t = *reinterpret_cast<const float4 *>(f.other + o);
            v.x = v.x + t.x;
            v.y = v.y + t.y;
            v.z = v.z + t.z;
            v.w = v.w + t.w;
        }
        const float4 a = *reinterpret_cast<const float4 *>(f.act + o);
        v.x = a.x > 0.0f ? v.x : 0.0f;
        v.y = a.y > 0.0f ? v.y : 0.0f;
        v.z = a.z > 0.0f ? v.z : 0.0f;
        v.w = a.w > 0.0f ? v.w : 0.0f;
    }
    return v;
}
