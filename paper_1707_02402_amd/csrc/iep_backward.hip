// Backward pass of an executed plan (paper: Results / IEP times the backward pass next to inference and
// expects the same gains from batching, since the pools are the same).  The launch groups are walked in
// reverse; inside a group every node is independent, and the gradients of the parameters are summed pool by
// pool (all nodes of one function in the group in one call), each parameter element by a single thread in item
// order, so the result does not depend on scheduling.
//
// For a node with residual block input u, mid = ReLU(conv_a(u) + b_a), y = ReLU(u + conv_b(mid) + b_b) and
// incoming gradient gy:
//     g    = gy * [y > 0]                      db_b += sum_p g      dW_b += g (x) mid
//     dmid = conv_b^T(g) * [mid > 0]           db_a += sum_p dmid   dW_a += dmid (x) u
//     du   = g + conv_a^T(dmid)
// and for a two-argument function, u = ReLU(conv1x1(concat(a0, a1)) + b1):
//     dc   = du * [u > 0]                      db_1 += sum_p dc     dW_1 += dc (x) concat
//     da0  = W1[:, :C]^T dc,  da1 = W1[:, C:]^T dc
// The node results y come from the forward pass (a plan made with DYNB_PLAN_KEEP leaves every one of them in the
// workspace); u of two-argument functions and mid are recomputed with the forward pass's generic kernels.
// Generic kernels: any shape, fp32 or bf16 values and weights, fp32 gradients, one thread per output element.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>
#include <vector>

#include "device_utils.h"
#include "iep_generic.h"
#include "plan_internal.h"

using dynb::fail;

#define HIP_TRY(expr, what)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(DYNB_E_HIP, std::string(what) + ": " + hipGetErrorString(e_));        \
    } while (0)

namespace {

struct BwdArgs {
    const dynb_item* items;       // the launch group's items
    const int32_t* gdst0;         // routes of the group's items
    const int32_t* gdst1;
    const uint8_t* arity;
    int32_t first_item;           // index of items[0] in the plan
    int32_t count;
    const void* feats;            // forward inputs / results
    const void* out;
    const void* slots;
    const void* tmp_u;            // recomputed, [count][HWC] storage type
    const void* tmp_m;
    const void* w1;
    const void* w3a;
    const void* w3b;
    float* gy;                    // [n_items][HWC]  gradient with respect to every item's result
    float* gleaf;                 // [n_leaves][HWC] gradient arriving at every SCENE leaf
    float* tmp_g;                 // [count][HWC]
    float* tmp_dm;                // [count][HWC]
    float* tmp_du;                // [count][HWC]
    int32_t C, H, W;
};

__device__ __forceinline__ float* route(const BwdArgs& a, int32_t r, size_t chw)
{
    return r >= 0 ? a.gy + size_t(r) * chw : a.gleaf + size_t(-1 - r) * chw;
}

// g = gy * [y > 0]
template <typename T>
__global__ void k_bwd_g(BwdArgs a)
{
    const int i = blockIdx.y;
    const dynb_item it = a.items[i];
    const size_t chw = size_t(a.H) * a.W * a.C;
    const size_t e = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= chw) return;
    const T* y = it.dst >= 0 ? (const T*)a.slots + size_t(it.dst) * chw : (const T*)a.out + size_t(-1 - it.dst) * chw;
    a.tmp_g[size_t(i) * chw + e] = load_f32(y + e) > 0.f ? a.gy[size_t(a.first_item + i) * chw + e] : 0.f;
}

// Transposed 3x3 convolution: r[q][ci] = sum_{co, kh, kw} gin[q - (kh-1, kw-1)][co] * w[t][co][kh][kw][ci]
// SECOND = false: gin = g, w = w3b, result masked by [mid > 0] -> tmp_dm
// SECOND = true:  gin = dmid, w = w3a, result + g = du -> the argument's gradient (one-argument functions) or tmp_du
template <typename T, bool SECOND>
__global__ void k_bwd_dgrad(BwdArgs a)
{
    const int i = blockIdx.y;
    const dynb_item it = a.items[i];
    const int C = a.C, H = a.H, W = a.W;
    const size_t chw = size_t(H) * W * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= int(chw)) return;
    const int q = e / C, ci = e % C, y = q / W, x = q % W;
    const float* gin = (SECOND ? a.tmp_dm : a.tmp_g) + size_t(i) * chw;
    const T* w = (const T*)(SECOND ? a.w3a : a.w3b) + size_t(it.type) * C * 9 * C;
    float acc = 0.f;
    for (int kh = 0; kh < 3; ++kh) {
        const int oy = y - (kh - 1);                  // the output pixel whose tap (kh, kw) reads input pixel q
        if (oy < 0 || oy >= H) continue;
        for (int kw = 0; kw < 3; ++kw) {
            const int ox = x - (kw - 1);
            if (ox < 0 || ox >= W) continue;
            const float* gp = gin + (size_t(oy) * W + ox) * C;
            const T* wk = w + size_t(kh * 3 + kw) * C + ci;
            for (int co = 0; co < C; ++co) acc += gp[co] * load_f32(wk + size_t(co) * 9 * C);
        }
    }
    if (!SECOND) {
        const float mid = load_f32((const T*)a.tmp_m + size_t(i) * chw + e);
        a.tmp_dm[size_t(i) * chw + e] = mid > 0.f ? acc : 0.f;
    } else {
        const float du = acc + a.tmp_g[size_t(i) * chw + e];
        if (a.arity[it.type] == 2) {
            const float u = load_f32((const T*)a.tmp_u + size_t(i) * chw + e);
            a.tmp_du[size_t(i) * chw + e] = u > 0.f ? du : 0.f;          // dc = du * [u > 0]
        } else {
            route(a, a.gdst0[i], chw)[e] = du;
        }
    }
}

// two-argument functions: da0[p][ci] = sum_co dc[p][co] * w1[co][ci], da1[p][ci] = sum_co dc[p][co] * w1[co][C + ci]
template <typename T>
__global__ void k_bwd_join(BwdArgs a)
{
    const int i = blockIdx.y;
    const dynb_item it = a.items[i];
    if (a.arity[it.type] != 2) return;
    const int C = a.C;
    const size_t chw = size_t(a.H) * a.W * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= int(chw)) return;
    const int p = e / C, ci = e % C;
    const float* dc = a.tmp_du + size_t(i) * chw + size_t(p) * C;
    const T* w = (const T*)a.w1 + size_t(it.type) * C * 2 * C;
    float s0 = 0.f, s1 = 0.f;
    for (int co = 0; co < C; ++co) {
        s0 += dc[co] * load_f32(w + size_t(co) * 2 * C + ci);
        s1 += dc[co] * load_f32(w + size_t(co) * 2 * C + C + ci);
    }
    route(a, a.gdst0[i], chw)[e] = s0;
    route(a, a.gdst1[i], chw)[e] = s1;
}

// Parameter gradients of one pool (items [lo, lo + n) of the group, all of function t).
// 3x3 weights: thread per element (co, kh, kw, ci):  dw += sum_items sum_p G[p][co] * IN[p + (kh-1, kw-1)][ci]
//   WHICH = 0: conv_b (G = g, IN = mid);  WHICH = 1: conv_a (G = dmid, IN = u)
template <typename T, int WHICH>
__global__ void k_bwd_wgrad3(BwdArgs a, int lo, int n, int t, float* __restrict__ dw)
{
    const int C = a.C, H = a.H, W = a.W;
    const size_t chw = size_t(H) * W * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= C * 9 * C) return;
    const int ci = e % C, tap = (e / C) % 9, co = e / (9 * C), kh = tap / 3, kw = tap % 3;
    float acc = 0.f;
    for (int i = lo; i < lo + n; ++i) {
        const float* G = (WHICH == 0 ? a.tmp_g : a.tmp_dm) + size_t(i) * chw;
        const T* IN;
        if (WHICH == 0) IN = (const T*)a.tmp_m + size_t(i) * chw;
        else {
            const dynb_item it = a.items[i];
            IN = a.arity[it.type] == 2 ? (const T*)a.tmp_u + size_t(i) * chw
                                       : (it.src0 >= 0 ? (const T*)a.slots + size_t(it.src0) * chw : (const T*)a.feats + size_t(-1 - it.src0) * chw);
        }
        for (int y = 0; y < H; ++y) {
            const int iy = y + kh - 1;
            if (iy < 0 || iy >= H) continue;
            for (int x = 0; x < W; ++x) {
                const int ix = x + kw - 1;
                if (ix < 0 || ix >= W) continue;
                acc += G[(size_t(y) * W + x) * C + co] * load_f32(IN + (size_t(iy) * W + ix) * C + ci);
            }
        }
    }
    dw[size_t(t) * C * 9 * C + e] += acc;
}

// biases of a pool: thread per channel; WHICH = 0: db_b from g, 1: db_a from dmid, 2: db_1 from dc
template <int WHICH>
__global__ void k_bwd_bias(BwdArgs a, int lo, int n, int t, float* __restrict__ db)
{
    const int C = a.C;
    const size_t P = size_t(a.H) * a.W, chw = P * C;
    const int co = blockIdx.x * blockDim.x + threadIdx.x;
    if (co >= C) return;
    const float* G = WHICH == 0 ? a.tmp_g : WHICH == 1 ? a.tmp_dm : a.tmp_du;
    float acc = 0.f;
    for (int i = lo; i < lo + n; ++i)
        for (size_t p = 0; p < P; ++p) acc += G[size_t(i) * chw + p * C + co];
    db[size_t(t) * C + co] += acc;
}

// 1x1 weights of a pool of two-argument functions: thread per (co, cj), cj over the 2C concatenated channels
template <typename T>
__global__ void k_bwd_wgrad1(BwdArgs a, int lo, int n, int t, float* __restrict__ dw)
{
    const int C = a.C;
    const size_t P = size_t(a.H) * a.W, chw = P * C;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= C * 2 * C) return;
    const int cj = e % (2 * C), co = e / (2 * C);
    float acc = 0.f;
    for (int i = lo; i < lo + n; ++i) {
        const dynb_item it = a.items[i];
        const int32_t s = cj < C ? it.src0 : it.src1;
        const T* in = s >= 0 ? (const T*)a.slots + size_t(s) * chw : (const T*)a.feats + size_t(-1 - s) * chw;
        const float* dc = a.tmp_du + size_t(i) * chw;
        const int c = cj < C ? cj : cj - C;
        for (size_t p = 0; p < P; ++p) acc += dc[p * C + co] * load_f32(in + p * C + c);
    }
    dw[size_t(t) * C * 2 * C + e] += acc;
}

__global__ void k_bwd_fill(float* p, size_t n, float v)
{
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += size_t(gridDim.x) * blockDim.x) p[i] = v;
}

// gy[root item of example e] = dout[e]
__global__ void k_bwd_seed(const float* __restrict__ dout, const int32_t* __restrict__ root_item, float* __restrict__ gy, size_t chw)
{
    const int e = blockIdx.y;
    const int32_t r = root_item[e];
    if (r < 0) return;
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < chw; i += size_t(gridDim.x) * blockDim.x)
        gy[size_t(r) * chw + i] = dout[size_t(e) * chw + i];
}

// dfeats[e] = sum of the gradients of e's SCENE leaves in leaf order; a program that is one SCENE token passes dout through
__global__ void k_bwd_leaves(const float* __restrict__ gleaf, const int32_t* __restrict__ leaf_first,
                             const int32_t* __restrict__ root_item, const float* __restrict__ dout, float* __restrict__ dfeats, size_t chw)
{
    const int e = blockIdx.y;
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < chw; i += size_t(gridDim.x) * blockDim.x) {
        float acc = 0.f;
        if (root_item[e] < 0) acc = dout[size_t(e) * chw + i];
        else
            for (int32_t l = leaf_first[e]; l < leaf_first[e + 1]; ++l) acc += gleaf[size_t(l) * chw + i];
        dfeats[size_t(e) * chw + i] = acc;
    }
}

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
size_t elt_bytes(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

struct BwdLayout {
    size_t gy, gleaf, tmp_u, tmp_m, tmp_g, tmp_dm, tmp_du, tables, total;
    size_t t_gdst0, t_gdst1, t_leaf_first, t_root_item;       // inside tables
};

BwdLayout bwd_layout(const dynb_plan* p, const dynb_shape* s)
{
    BwdLayout L;
    const size_t chw = size_t(s->C) * s->H * s->W, n_items = p->items.size();
    const size_t n_leaf = p->leaf_first.empty() ? 0 : size_t(p->leaf_first.back());
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(std::max<size_t>(bytes, 4)); return at; };
    L.gy = take(n_items * chw * 4);
    L.gleaf = take(n_leaf * chw * 4);
    L.tmp_u = take(size_t(p->max_launch) * chw * elt_bytes(s->dtype));
    L.tmp_m = take(size_t(p->max_launch) * chw * elt_bytes(s->dtype));
    L.tmp_g = take(size_t(p->max_launch) * chw * 4);
    L.tmp_dm = take(size_t(p->max_launch) * chw * 4);
    L.tmp_du = take(size_t(p->max_launch) * chw * 4);
    L.tables = o;
    L.t_gdst0 = take(n_items * 4);
    L.t_gdst1 = take(n_items * 4);
    L.t_leaf_first = take((size_t(p->B) + 1) * 4);
    L.t_root_item = take(size_t(p->B) * 4);
    L.total = o;
    return L;
}

template <typename T>
int run_backward(const dynb_plan* p, const dynb_shape* s, const dynb_module_weights* w, const void* feats, const void* out,
                 const void* fwd_ws, const float* dout, const dynb_module_grads* g, char* ws, hipStream_t st)
{
    const BwdLayout L = bwd_layout(p, s);
    const size_t chw = size_t(s->C) * s->H * s->W;
    const int C = s->C, B = p->B;
    // the routing tables travel with the call (a few bytes per node)
    auto table = [&](size_t at, const std::vector<int32_t>& v) -> hipError_t {
        return v.empty() ? hipSuccess : hipMemcpyAsync(ws + at, v.data(), v.size() * 4, hipMemcpyHostToDevice, st);
    };
    HIP_TRY(table(L.t_gdst0, p->grad_dst0), "dynbatch_backward(tables)");
    HIP_TRY(table(L.t_gdst1, p->grad_dst1), "dynbatch_backward(tables)");
    HIP_TRY(table(L.t_leaf_first, p->leaf_first), "dynbatch_backward(tables)");
    HIP_TRY(table(L.t_root_item, p->root_item), "dynbatch_backward(tables)");
    const int32_t* d_leaf_first = reinterpret_cast<const int32_t*>(ws + L.t_leaf_first);
    const int32_t* d_root_item = reinterpret_cast<const int32_t*>(ws + L.t_root_item);

    auto fill = [&](float* ptr, size_t n) {
        if (ptr && n) hipLaunchKernelGGL(k_bwd_fill, dim3(unsigned(std::min<size_t>((n + 255) / 256, 4096))), dim3(256), 0, st, ptr, n, 0.f);
    };
    const size_t nt = size_t(p->n_types);
    fill(g->dw3a, nt * C * 9 * C); fill(g->dw3b, nt * C * 9 * C); fill(g->db3a, nt * C); fill(g->db3b, nt * C);
    fill(g->dw1, nt * C * 2 * C); fill(g->db1, nt * C);

    float* gy = reinterpret_cast<float*>(ws + L.gy);
    const unsigned bx_map = unsigned(std::min<size_t>((chw + 255) / 256, 64));
    for (int e0 = 0; e0 < B; e0 += 32768)
        hipLaunchKernelGGL(k_bwd_seed, dim3(bx_map, unsigned(std::min(32768, B - e0))), dim3(256), 0, st, dout + size_t(e0) * chw,
                           d_root_item + e0, gy, chw);

    const char* d = static_cast<const char*>(p->dev_buf);
    const dynb_item* d_items = reinterpret_cast<const dynb_item*>(d);
    const uint8_t* d_arity = reinterpret_cast<const uint8_t*>(d + dynb_plan_arity_offset(p));
    GenArgs ga;                                     // recomputation of u and mid with the forward kernels
    ga.arity = d_arity;
    ga.feats = feats; ga.out = nullptr; ga.slots = const_cast<void*>(fwd_ws);
    ga.w1 = w->w1; ga.b1 = w->b1; ga.w3a = w->w3a; ga.b3a = w->b3a; ga.w3b = w->w3b; ga.b3b = w->b3b;
    ga.C = s->C; ga.H = s->H; ga.W = s->W;
    BwdArgs ba;
    ba.arity = d_arity;
    ba.feats = feats; ba.out = out; ba.slots = fwd_ws;
    ba.w1 = w->w1; ba.w3a = w->w3a; ba.w3b = w->w3b;
    ba.gy = gy; ba.gleaf = reinterpret_cast<float*>(ws + L.gleaf);
    ba.C = s->C; ba.H = s->H; ba.W = s->W;
    const unsigned bx = unsigned((chw + 255) / 256);
    const unsigned bw3 = unsigned((size_t(C) * 9 * C + 255) / 256), bw1 = unsigned((size_t(C) * 2 * C + 255) / 256), bb = unsigned((C + 255) / 256);

    for (size_t li = p->launches.size(); li-- > 0;) {
        const dynb_launch& l = p->launches[li];
        // a launch group wider than one grid (65535 rows) is walked in slices; its nodes are independent
        for (int off = 0; off < l.count; off += 32768) {
            const int cnt = std::min(32768, l.count - off);
            const int first = l.start + off;
            ga.items = d_items + first; ga.count = cnt;
            ga.tmp_u = ws + L.tmp_u; ga.tmp_m = ws + L.tmp_m;
            ba.items = d_items + first; ba.first_item = first; ba.count = cnt;
            ba.gdst0 = reinterpret_cast<const int32_t*>(ws + L.t_gdst0) + first;
            ba.gdst1 = reinterpret_cast<const int32_t*>(ws + L.t_gdst1) + first;
            ba.tmp_u = ws + L.tmp_u; ba.tmp_m = ws + L.tmp_m;
            ba.tmp_g = reinterpret_cast<float*>(ws + L.tmp_g); ba.tmp_dm = reinterpret_cast<float*>(ws + L.tmp_dm);
            ba.tmp_du = reinterpret_cast<float*>(ws + L.tmp_du);
            const dim3 grid(bx, unsigned(cnt));
            if (l.any_binary) hipLaunchKernelGGL((k_gen_join<T>), grid, dim3(256), 0, st, ga);
            hipLaunchKernelGGL((k_gen_conv<T, false>), grid, dim3(256), 0, st, ga);
            hipLaunchKernelGGL((k_bwd_g<T>), grid, dim3(256), 0, st, ba);
            hipLaunchKernelGGL((k_bwd_dgrad<T, false>), grid, dim3(256), 0, st, ba);
            hipLaunchKernelGGL((k_bwd_dgrad<T, true>), grid, dim3(256), 0, st, ba);
            if (l.any_binary) hipLaunchKernelGGL((k_bwd_join<T>), grid, dim3(256), 0, st, ba);
            // parameter gradients, pool by pool: runs of equal function id (the items of a group are sorted by function)
            int lo = 0;
            while (lo < cnt) {
                const int t = p->items[first + lo].type;
                int n = 1;
                while (lo + n < cnt && p->items[first + lo + n].type == t) ++n;
                hipLaunchKernelGGL((k_bwd_wgrad3<T, 0>), dim3(bw3), dim3(256), 0, st, ba, lo, n, t, g->dw3b);
                hipLaunchKernelGGL((k_bwd_wgrad3<T, 1>), dim3(bw3), dim3(256), 0, st, ba, lo, n, t, g->dw3a);
                hipLaunchKernelGGL((k_bwd_bias<0>), dim3(bb), dim3(256), 0, st, ba, lo, n, t, g->db3b);
                hipLaunchKernelGGL((k_bwd_bias<1>), dim3(bb), dim3(256), 0, st, ba, lo, n, t, g->db3a);
                if (p->arity[t] == 2) {
                    hipLaunchKernelGGL((k_bwd_wgrad1<T>), dim3(bw1), dim3(256), 0, st, ba, lo, n, t, g->dw1);
                    hipLaunchKernelGGL((k_bwd_bias<2>), dim3(bb), dim3(256), 0, st, ba, lo, n, t, g->db1);
                }
                lo += n;
            }
        }
    }
    for (int e0 = 0; e0 < B; e0 += 32768)
        hipLaunchKernelGGL(k_bwd_leaves, dim3(bx_map, unsigned(std::min(32768, B - e0))), dim3(256), 0, st, ba.gleaf, d_leaf_first + e0,
                           d_root_item + e0, dout + size_t(e0) * chw, g->dfeats + size_t(e0) * chw, chw);
    HIP_TRY(hipGetLastError(), "dynbatch_backward");
    return DYNB_OK;
}

int check_backward(const dynb_plan* p, const dynb_shape* s, const char* who)
{
    if (!p || !s) return fail(DYNB_E_INVAL, std::string(who) + ": NULL argument");
    if (s->C <= 0 || s->H <= 0 || s->W <= 0) return fail(DYNB_E_INVAL, std::string(who) + ": C, H, W must be positive");
    if (s->dtype != DYNB_F32 && s->dtype != DYNB_BF16) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": unknown dtype");
    if (!p->keep) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": the plan was not made with DYNB_PLAN_KEEP");
    if (p->shared_nodes) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": dependency graphs with shared nodes have no backward pass yet");
    if (size_t(s->C) * s->H * s->W >= (size_t(1) << 31) || size_t(s->C) * 9 * s->C >= (size_t(1) << 31))
        return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": map too large");
    return DYNB_OK;
}

}  // namespace

extern "C" size_t dynbatch_backward_workspace_bytes(const dynb_plan* p, const dynb_shape* s)
{
    if (check_backward(p, s, "dynbatch_backward_workspace_bytes") != DYNB_OK) return 0;
    return std::max<size_t>(bwd_layout(p, s).total, 256);
}

extern "C" int dynbatch_backward(const dynb_plan* p, const dynb_shape* s, const dynb_module_weights* w, const void* feats,
                                 const void* out, const void* forward_workspace, const float* dout,
                                 const dynb_module_grads* grads, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_backward(p, s, "dynbatch_backward");
    if (rc != DYNB_OK) return rc;
    if (!w || !feats || !out || !forward_workspace || !dout || !grads || !workspace)
        return fail(DYNB_E_INVAL, "dynbatch_backward: NULL argument");
    if (!w->w3a || !w->w3b) return fail(DYNB_E_INVAL, "dynbatch_backward: conv3x3 weights missing");
    if (!grads->dfeats || !grads->dw3a || !grads->db3a || !grads->dw3b || !grads->db3b)
        return fail(DYNB_E_INVAL, "dynbatch_backward: a gradient tensor is missing");
    if (p->has_binary && (!w->w1 || !grads->dw1 || !grads->db1))
        return fail(DYNB_E_INVAL, "dynbatch_backward: two-argument functions need w1, dw1 and db1");
    if (!p->dev_buf) return fail(DYNB_E_WORKSPACE, "dynbatch_backward: plan not uploaded");
    if (workspace_bytes < bwd_layout(p, s).total) return fail(DYNB_E_WORKSPACE, "dynbatch_backward: workspace too small");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(DYNB_E_INVAL, "dynbatch_backward: workspace not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    if (s->dtype == DYNB_BF16) return run_backward<bf16_t>(p, s, w, feats, out, forward_workspace, dout, grads, ws, st);
    return run_backward<float>(p, s, w, feats, out, forward_workspace, dout, grads, ws, st);
}
