// Generic kernels of the program-tree executor: any C/H/W, fp32 or bf16 storage, fp32 accumulation, one thread
// per output element.  Shared by the forward executor (shapes without a fused MFMA kernel) and by the backward
// pass (which recomputes a module's inner activations with them).
#pragma once

#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "plan_internal.h"

namespace {

// ------------------------------------------------------------------------------------------
// Generic kernels
// ------------------------------------------------------------------------------------------
struct GenArgs {
    const dynb_item* items;
    const uint8_t* arity;     // device [n_types]
    int32_t count;
    const void* feats;
    void* out;
    void* slots;
    void* tmp_u;
    void* tmp_m;
    const void* w1;
    const float* b1;
    const void* w3a;
    const float* b3a;
    const void* w3b;
    const float* b3b;
    int32_t C, H, W;
};

template <typename T>
__device__ __forceinline__ const T* src_map(const GenArgs& a, int32_t s, size_t chw)
{
    return s >= 0 ? (const T*)a.slots + size_t(s) * chw : (const T*)a.feats + size_t(-1 - s) * chw;
}

// u = ReLU(conv1x1(concat(arg0, arg1)) + b1) for the binary items of a launch group
template <typename T>
__global__ void k_gen_join(GenArgs a)
{
    const int i = blockIdx.y;
    const dynb_item it = a.items[i];
    if (a.arity[it.type] != 2) return;
    const int C = a.C;
    const size_t chw = size_t(a.H) * a.W * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= int(chw)) return;
    const int p = e / C, co = e % C;
    const T* x0 = src_map<T>(a, it.src0, chw) + size_t(p) * C;
    const T* x1 = src_map<T>(a, it.src1, chw) + size_t(p) * C;
    const T* w = (const T*)a.w1 + (size_t(it.type) * C + co) * 2 * C;
    float acc = a.b1 ? a.b1[size_t(it.type) * C + co] : 0.f;
    for (int ci = 0; ci < C; ++ci) acc += load_f32(x0 + ci) * load_f32(w + ci);
    for (int ci = 0; ci < C; ++ci) acc += load_f32(x1 + ci) * load_f32(w + C + ci);
    store_f32((T*)a.tmp_u + size_t(i) * chw + e, fmaxf(acc, 0.f));
}

// SECOND = false: mid = ReLU(conv3x3_a(u) + b3a);  SECOND = true: y = ReLU(u + conv3x3_b(mid) + b3b)
template <typename T, bool SECOND>
__global__ void k_gen_conv(GenArgs a)
{
    const int i = blockIdx.y;
    const dynb_item it = a.items[i];
    const int C = a.C, H = a.H, W = a.W;
    const size_t chw = size_t(H) * W * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= int(chw)) return;
    const int p = e / C, co = e % C, y = p / W, x = p % W;
    const T* u = (a.arity[it.type] == 2) ? (const T*)a.tmp_u + size_t(i) * chw : src_map<T>(a, it.src0, chw);
    const T* in = SECOND ? (const T*)a.tmp_m + size_t(i) * chw : u;
    const T* w = (const T*)(SECOND ? a.w3b : a.w3a) + (size_t(it.type) * C + co) * 9 * C;
    const float* b = SECOND ? a.b3b : a.b3a;
    float acc = b ? b[size_t(it.type) * C + co] : 0.f;
    for (int kh = 0; kh < 3; ++kh) {
        const int iy = y + kh - 1;
        if (iy < 0 || iy >= H) continue;
        for (int kw = 0; kw < 3; ++kw) {
            const int ix = x + kw - 1;
            if (ix < 0 || ix >= W) continue;
            const T* px = in + (size_t(iy) * W + ix) * C;
            const T* wk = w + (kh * 3 + kw) * C;
            for (int ci = 0; ci < C; ++ci) acc += load_f32(px + ci) * load_f32(wk + ci);
        }
    }
    if (!SECOND) {
        store_f32((T*)a.tmp_m + size_t(i) * chw + e, fmaxf(acc, 0.f));
    } else {
        acc += load_f32(u + e);
        T* dst = it.dst >= 0 ? (T*)a.slots + size_t(it.dst) * chw : (T*)a.out + size_t(-1 - it.dst) * chw;
        store_f32(dst + e, fmaxf(acc, 0.f));
    }
}

}  // namespace
