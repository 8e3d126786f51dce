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
// Two kernel families with the same semantics, like the forward pass: MFMA kernels for bf16, C = 128, 14 x 14 (further
// down), and generic kernels for any shape, fp32 or bf16 values and weights, fp32 gradients, one thread per output
// element, which recompute u and mid with the forward pass's generic kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <string>
#include <type_traits>
#include <vector>

#include "device_utils.h"
#include "iep_generic.h"
#include "iep_mfma.h"
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

// ------------------------------------------------------------------------------------------
// MFMA path: bf16, C = 128, 14 x 14 (the shape of the fused forward kernel)
// ------------------------------------------------------------------------------------------
// The transposed convolutions are convolutions with the taps flipped and the channel roles exchanged, so a node's
// backward step has the shape of its forward step and runs on the same building blocks (LDS halo tile, packed
// weight fragments, software-pipelined K loop), one node per workgroup, wave w owning channel tile w.  The forward
// pass of a DYNB_PLAN_KEEP plan has left u (two-argument functions) and mid of every item in its workspace.
//   tile <- g = gy * [y > 0]   (bf16)
//   conv(g; W_b flipped^T)     -> dmid = result * [mid > 0], written into the tile in place of g
//   conv(dmid; W_a flipped^T)  -> du = that + g (the residual path, in fp32 from the gradient map), written as fp32
//                                 to the argument's gradient map; two-argument functions: dc = du * [u > 0] into the
//                                 tile, then two 1x1 convolutions with the halves of W_1^T
// Everything that enters or leaves in the accumulator layout (masks, the residual term, results) goes through LDS so
// that all global accesses are coalesced 16-byte pieces.
// Gradients travel between nodes as fp32 maps and enter the MFMAs as bf16 (like every other operand of this
// path).  g, dmid and dc are saved as bf16 maps per item for the parameter gradients, which one kernel sums
// function by function afterwards.
struct BmArgs {
    const dynb_item* items;       // the launch group's items
    const int32_t* gdst0;         // routes of the group's items
    const int32_t* gdst1;
    const uint8_t* arity;
    int32_t first_item;
    int32_t count;
    const bf16_t* feats;
    const bf16_t* out;
    const bf16_t* slots;
    const bf16_t* pk3bT;          // packed fragments: conv_b, taps flipped, channels exchanged
    const bf16_t* pk3aT;          //                   conv_a, taps flipped, channels exchanged
    const bf16_t* pk1T;           //                   conv1x1 halves, channels exchanged
    float* gy;                    // [n_items][P*C]
    float* gleaf;                 // [n_leaves][P*C]
    const bf16_t* sv_u;           // [n_items][P*C] each; u and mid: in the forward pass's workspace
    const bf16_t* sv_m;
    bf16_t* sv_g;
    bf16_t* sv_dm;
    bf16_t* sv_dc;
};

// a bf16 is positive iff its bits, read as int16, are positive; for the two halves of a packed pair
__device__ __forceinline__ bool bf16_lo_positive(uint32_t w) { return int16_t(w & 0xffffu) > 0; }
__device__ __forceinline__ bool bf16_hi_positive(uint32_t w) { return int16_t(w >> 16) > 0; }

__device__ __forceinline__ float* route_mf(const BmArgs& a, int32_t r)
{
    return r >= 0 ? a.gy + size_t(r) * (mf::P * mf::C) : a.gleaf + size_t(-1 - r) * (mf::P * mf::C);
}

// dst[function][tile][tap][j][lane][i] = W(o, tap, k) with o = tile*32 + rho(lane % 32) (the row permutation of the
// forward pass's packed weights), k = (lane/32)*64 + j*8 + i, where
//   mode 0: W = src[function][o][tap][k]                 conv3x3 as given (ntap 9)
//   mode 1: W = src[function][k][8 - tap][o]             conv3x3 transposed, taps flipped (ntap 9)
//   mode 2: W = src[function][o][tap*128 + k]            conv1x1 over 2C inputs, half `tap` (ntap 2)
//   mode 3: W = src[function][k][tap*128 + o]            conv1x1 transposed, half `tap` (ntap 2)
__global__ void k_bwd_pack(const bf16_t* __restrict__ src, u32x4* __restrict__ dst, int n_types, int ntap, int mode)
{
    const size_t total = size_t(n_types) * 4 * ntap * 8 * 64;
    for (size_t q = size_t(blockIdx.x) * blockDim.x + threadIdx.x; q < total; q += size_t(gridDim.x) * blockDim.x) {
        const int lane = int(q & 63), j = int((q >> 6) & 7);
        const size_t rest = q >> 9;
        const int tap = int(rest % ntap), tile = int((rest / ntap) & 3);
        const size_t type = rest / (size_t(ntap) * 4);
        const int m = lane & 31;
        const int o = tile * 32 + ((m >> 2) & 1) * 16 + (m >> 3) * 4 + (m & 3), k0 = (lane >> 5) * 64 + j * 8;
        uint32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = k0 + i;
            size_t e;
            if (mode == 0) e = ((type * 128 + o) * 9 + tap) * 128 + k;
            else if (mode == 1) e = ((type * 128 + k) * 9 + (8 - tap)) * 128 + o;
            else if (mode == 2) e = (type * 128 + o) * 256 + tap * 128 + k;
            else e = (type * 128 + k) * 256 + tap * 128 + o;
            v[i] = src[e];
        }
        dst[q] = u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
    }
}

// LDS of the backward node kernel: the halo tile, one mask byte per 16-byte piece of the y and the mid map, and an
// fp32 staging area through which accumulators (lane = pixel) leave as coalesced 16-byte pieces.  A global access in
// which every lane touches a line of its own costs about 125 clocks to issue, so nothing is loaded or stored in the
// accumulator layout: masks come from the LDS bytes, the residual term and the result go through the staging area.
namespace bn {
constexpr int MASK_OFF = mf::TILE_BYTES;                 // y mask bytes [P][16], then mid mask bytes [P][16]
constexpr int MASK_BYTES = 2 * mf::P * 16 + 128;         // (+ padding to a multiple of 256)
constexpr int STAGE_OFF = MASK_OFF + MASK_BYTES;
constexpr int STAGE_PITCH = mf::C * 4 + 16;              // bytes per pixel: 128 floats + a bank-shifting pad
constexpr int STAGE_PIX = 128;                           // pixels per round: four pixel tiles
constexpr int LDS_BYTES = STAGE_OFF + STAGE_PIX * STAGE_PITCH;
static_assert(MASK_BYTES % 256 == 0 && LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
}  // namespace bn

template <int RW>
__global__ __launch_bounds__(256, 1) void k_bwd_node_mfma(BmArgs a)
{
    using namespace mf;
    constexpr int MTW = MT7, NT = 1, XS = 4, NTHR = 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= a.count) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, h = lane >> 5, n0 = wave * 32;
#ifdef DYNB_NODE_CLOCKS
    long long tck[10], tck0 = clock64();
#define NCLK(i) tck[i] = clock64() - tck0
#else
#define NCLK(i) do {} while (0)
#endif
    const dynb_item it = a.items[logical];
    const bool binary = a.arity[it.type] == 2;                        // uniform over the workgroup
    const size_t item_off = size_t(a.first_item + logical) * (P * C);

    const size_t frag3 = (size_t(it.type) * 4 + wave) * 9 * 8, frag1 = (size_t(it.type) * 4 + wave) * 2 * 8;
    const bf16_t* wrow_bT[NT] = {a.pk3bT + frag3 * FRAG + lane * 8};
    const bf16_t* wrow_aT[NT] = {a.pk3aT + frag3 * FRAG + lane * 8};
    bf16x8 ring[RW][NT];

    auto centre_addr = [&](int c) -> uint32_t {                       // 16-byte piece c of a map -> its place in the halo tile
        const int p = c >> 4, part = c & 15;
        return uint32_t((p / S + 1) * ROW_BYTES + (p % S + 1) * PIX_BYTES + part * 16);
    };
    // bit i of the result: element i of the piece is positive
    auto piece_mask = [](const u32x4& v) -> uint32_t {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t bits = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) bits |= (bf16_lo_positive(w[i]) ? 1u : 0u) << (2 * i) | (bf16_hi_positive(w[i]) ? 1u : 0u) << (2 * i + 1);
        return bits;
    };
    const float* gyp = a.gy + item_off;
    const bf16_t* yp = it.dst >= 0 ? a.slots + size_t(it.dst) * (P * C) : a.out + size_t(-1 - it.dst) * (P * C);

    // ---- g = gy * [y > 0] as bf16 into the tile, saved for dW_b and db_b; mask bytes of y and mid; all loads are
    // issued before the first use
    constexpr int NIT = (P * 16 + NTHR - 1) / NTHR;
    {
        const f32x4* gy4 = reinterpret_cast<const f32x4*>(gyp);
        const u32x4* y4 = reinterpret_cast<const u32x4*>(yp);
        u32x4* sg4 = reinterpret_cast<u32x4*>(a.sv_g + item_off);
        f32x4 glo[NIT], ghi[NIT];
        u32x4 yv[NIT];
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tid + i * NTHR;
            if (c < P * 16) { glo[i] = gy4[2 * c]; ghi[i] = gy4[2 * c + 1]; yv[i] = y4[c]; }
        }
        __builtin_amdgcn_sched_barrier(0);
        ring_fill<NT, RW>(ring, wrow_bT);                             // arrives while the tile is written
        for (int c = tid; c < 60 * 16; c += NTHR) {                   // zero border
            const int q = c >> 4, part = c & 15;
            int row, col;
            if (q < 16) { row = 0; col = q; }
            else if (q < 32) { row = HALO - 1; col = q - 16; }
            else { row = 1 + ((q - 32) >> 1); col = ((q - 32) & 1) ? HALO - 1 : 0; }
            *reinterpret_cast<u32x4*>(lds_raw + uint32_t(row * ROW_BYTES + col * PIX_BYTES + part * 16)) = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tid + i * NTHR;
            if (c < P * 16) {
                const uint32_t yb = piece_mask(yv[i]);
                u32x4 pk;
                pk.x = pack_bf16x2(yb & 1u ? glo[i].x : 0.f, yb & 2u ? glo[i].y : 0.f);
                pk.y = pack_bf16x2(yb & 4u ? glo[i].z : 0.f, yb & 8u ? glo[i].w : 0.f);
                pk.z = pack_bf16x2(yb & 16u ? ghi[i].x : 0.f, yb & 32u ? ghi[i].y : 0.f);
                pk.w = pack_bf16x2(yb & 64u ? ghi[i].z : 0.f, yb & 128u ? ghi[i].w : 0.f);
                *reinterpret_cast<u32x4*>(lds_raw + centre_addr(c)) = pk;
                sg4[c] = pk;
                lds_raw[bn::MASK_OFF + c] = static_cast<unsigned char>(yb);
            }
        }
    }

    uint32_t xaddr[MTW];                                              // top-left tap of this lane's pixel, its 64-channel half
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        const int p = min(t * 32 + r, P - 1);
        xaddr[t] = uint32_t((p / S) * ROW_BYTES + (p % S) * PIX_BYTES + h * 128);
    }
    const int chan = n0 + 16 * h;                                     // this lane's 16 accumulator elements: channels chan .. chan+15
    f32x16 acc[MTW][NT];
    auto zero_acc = [&]() {
#pragma unroll
        for (int t = 0; t < MTW; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][0][i] = 0.f;
    };
    auto centre = [&](int t) -> uint32_t { return xaddr[t] - uint32_t(h * 128) + CENTER; };
    // acc[t][0][8q .. 8q+7] where the mask bit is set, as 8 packed bf16
    auto packed_masked = [&](int t, int q, uint32_t bits) -> u32x4 {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (bits >> (8 * q + i)) & 1u ? acc[t][0][8 * q + i] : 0.f;
        return u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    };
    // Accumulators -> the fp32 staging area, four pixel tiles per round; then every thread takes 16-byte pieces
    // (8 channels of a pixel) out of it: fn(c, lo, hi, pre(c)) with c the piece's index in the whole map.  pre(c)
    // is evaluated for all of a thread's pieces before the round's barriers, so what it loads is there afterwards.
    auto through_lds = [&](auto&& pre, auto&& fn) {
#pragma unroll
        for (int round = 0; round < 2; ++round) {
            const int t0 = round * 4, t1 = round == 0 ? 4 : MTW, p0 = t0 * 32, p1 = round == 0 ? 128 : P;
            constexpr int NI = 128 * 16 / NTHR;                       // pieces per thread of the larger round
            decltype(pre(0)) ahead[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int c = p0 * 16 + tid + i * NTHR;
                if (c < p1 * 16) ahead[i] = pre(c);
            }
            __syncthreads();                                          // the area (and, the first time, the tile) is free
#pragma unroll
            for (int t = 0; t < MTW; ++t)
                if (t >= t0 && t < t1) {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        *reinterpret_cast<f32x4*>(lds_raw + bn::STAGE_OFF + uint32_t(((t - t0) * 32 + r) * bn::STAGE_PITCH + (chan + 4 * b) * 4)) =
                            f32x4{acc[t][0][4 * b], acc[t][0][4 * b + 1], acc[t][0][4 * b + 2], acc[t][0][4 * b + 3]};
                }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int c = p0 * 16 + tid + i * NTHR;
                if (c < p1 * 16) {
                    const uint32_t at = bn::STAGE_OFF + uint32_t(((c >> 4) - p0) * bn::STAGE_PITCH + (c & 15) * 32);
                    fn(c, *reinterpret_cast<const f32x4*>(lds_raw + at), *reinterpret_cast<const f32x4*>(lds_raw + at + 16), ahead[i]);
                }
            }
        }
    };
    struct Nothing {};
    struct Grad { f32x4 g0, g1; };
    struct GradU { f32x4 g0, g1; u32x4 u; };
    auto store_piece = [](float* dst, int c, const f32x4& lo, const f32x4& hi) {
        *reinterpret_cast<f32x4*>(dst + size_t(c) * 8) = lo;
        *reinterpret_cast<f32x4*>(dst + size_t(c) * 8 + 4) = hi;
    };
    NCLK(0);
    __syncthreads();

    // ---- dmid = conv(g; W_b flipped, transposed) * [mid > 0], written into the tile in place of g
    // (mid is requested now and turned into mask bytes after the loop)
    u32x4 mv[NIT];
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int c = tid + i * NTHR;
        if (c < P * 16) mv[i] = reinterpret_cast<const u32x4*>(a.sv_m + item_off)[c];
    }
    zero_acc();
    NCLK(1);
    kloop<MTW, NT, RW, XS, false>(acc, xaddr, ring, wrow_bT, wrow_aT);
    NCLK(2);
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int c = tid + i * NTHR;
        if (c < P * 16) lds_raw[bn::MASK_OFF + P * 16 + c] = static_cast<unsigned char>(piece_mask(mv[i]));
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MTW; ++t)
        if (t * 32 + r < P) {
            // this lane's 16 mask bits: the bytes of the two pieces that hold its channels
            const uint32_t mm = *reinterpret_cast<const uint16_t*>(lds_raw + bn::MASK_OFF + P * 16 + (t * 32 + r) * 16 + (chan >> 3));
#pragma unroll
            for (int q = 0; q < 2; ++q)
                *reinterpret_cast<u32x4*>(lds_raw + centre(t) + uint32_t((chan + q * 8) * 2)) = packed_masked(t, q, mm);
        }
    __syncthreads();
    {                                                                 // dmid saved for dW_a and db_a, out of the tile
        u32x4* sdm4 = reinterpret_cast<u32x4*>(a.sv_dm + item_off);
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tid + i * NTHR;
            if (c < P * 16) sdm4[c] = *reinterpret_cast<const u32x4*>(lds_raw + centre_addr(c));
        }
    }

    // ---- du = g + conv(dmid; W_a flipped, transposed).  The residual term g is added in fp32, from the gradient map
    // itself, not from its bf16 copy in the tile: down a chain of modules the convolution's share is small against
    // the residual's and would vanish below the bfloat16 quantum of the latter at every level.
    zero_acc();
    NCLK(3);
    kloop<MTW, NT, RW, XS, false>(acc, xaddr, ring, wrow_aT, wrow_aT);
    NCLK(4);
    auto residual = [&](int c, f32x4& lo, f32x4& hi, const f32x4& g0, const f32x4& g1) {
        const uint32_t yb = lds_raw[bn::MASK_OFF + c];
        lo.x += yb & 1u ? g0.x : 0.f; lo.y += yb & 2u ? g0.y : 0.f; lo.z += yb & 4u ? g0.z : 0.f; lo.w += yb & 8u ? g0.w : 0.f;
        hi.x += yb & 16u ? g1.x : 0.f; hi.y += yb & 32u ? g1.y : 0.f; hi.z += yb & 64u ? g1.z : 0.f; hi.w += yb & 128u ? g1.w : 0.f;
    };
    const f32x4* gy4 = reinterpret_cast<const f32x4*>(gyp);
    if (!binary) {
        float* dst = route_mf(a, a.gdst0[logical]);
        through_lds([&](int c) { return Grad{gy4[2 * c], gy4[2 * c + 1]}; },
                    [&](int c, f32x4 lo, f32x4 hi, const Grad& g) {
                        residual(c, lo, hi, g.g0, g.g1);
                        store_piece(dst, c, lo, hi);
                    });
        NCLK(5);
#ifdef DYNB_NODE_CLOCKS
        if (logical == 0 && (threadIdx.x & 63) == 0)
            printf("node count %d wave %d: staged %lld | conv1 %lld..%lld | conv2 %lld..%lld | stored %lld\n", a.count, int(threadIdx.x >> 6), tck[0],
                   tck[1], tck[2], tck[3], tck[4], tck[5]);
#endif
        return;
    }
    // ---- two-argument functions: dc = du * [u > 0] into the tile, then da0 = dc W_1[:, :C], da1 = dc W_1[:, C:]
    {
        const u32x4* u4 = reinterpret_cast<const u32x4*>(a.sv_u + item_off);
        u32x4* sdc4 = reinterpret_cast<u32x4*>(a.sv_dc + item_off);
        through_lds([&](int c) { return GradU{gy4[2 * c], gy4[2 * c + 1], u4[c]}; },
                    [&](int c, f32x4 lo, f32x4 hi, const GradU& g) {
                        residual(c, lo, hi, g.g0, g.g1);
                        const uint32_t ub = piece_mask(g.u);
                        u32x4 pk;
                        pk.x = pack_bf16x2(ub & 1u ? lo.x : 0.f, ub & 2u ? lo.y : 0.f);
                        pk.y = pack_bf16x2(ub & 4u ? lo.z : 0.f, ub & 8u ? lo.w : 0.f);
                        pk.z = pack_bf16x2(ub & 16u ? hi.x : 0.f, ub & 32u ? hi.y : 0.f);
                        pk.w = pack_bf16x2(ub & 64u ? hi.z : 0.f, ub & 128u ? hi.w : 0.f);
                        *reinterpret_cast<u32x4*>(lds_raw + centre_addr(c)) = pk;
                        sdc4[c] = pk;
                    });
    }
    __syncthreads();
    {
        const bf16_t* t1row[NT] = {a.pk1T + frag1 * FRAG + lane * 8};
        const bf16_t* t1row2[NT] = {t1row[0] + 8 * FRAG};
        bf16x8 ring1[8][NT];
        ring_fill<NT, 8>(ring1, t1row);
        zero_acc();
        kloop<MTW, NT, 8, XS, true>(acc, xaddr, ring1, t1row, t1row2);
        float* d0 = route_mf(a, a.gdst0[logical]);
        through_lds([](int) { return Nothing{}; }, [&](int c, f32x4 lo, f32x4 hi, const Nothing&) { store_piece(d0, c, lo, hi); });
        zero_acc();
        kloop<MTW, NT, 8, XS, true>(acc, xaddr, ring1, t1row2, t1row2);
        float* d1 = route_mf(a, a.gdst1[logical]);
        through_lds([](int) { return Nothing{}; }, [&](int c, f32x4 lo, f32x4 hi, const Nothing&) { store_piece(d1, c, lo, hi); });
    }
}

// Parameter gradients.  A unit of work sums one chunk of a function's items for one (mode, part):
//   mode 0: conv_b, part = kernel row kh:  dW_b[co][kh][kw][ci] = sum_items sum_p g[p][co]    mid[p + (kh-1, kw-1)][ci]
//   mode 1: conv_a, part = kernel row kh:  dW_a[co][kh][kw][ci] = sum_items sum_p dmid[p][co] u[p + (kh-1, kw-1)][ci]
//   mode 2: conv1x1, part = argument:      dW_1[co][part*C + ci] = sum_items sum_p dc[p][co]  arg_part[p][ci]
// and with part 0 the bias gradient, the sum of g / dmid / dc over items and pixels.
// The contraction runs over pixels, the dimension in which neither map is contiguous.  Both maps of an item are
// copied into LDS halo tiles (pixel-major like the forward pass's tile) and the MFMA operands are read from
// there four bytes (two channels of a pixel) at a time: lane (m, hk) holds, for the 8 pixels x = 8 hk .. 8 hk + 7 of image
// row y, channels 2 m and 2 m + 1, which are row m of the wave's two interleaved channel tiles; a K step is an image
// row (x = 14, 15 are zeros).  For a kernel row the three taps' fragments of the
// input map are the same 10 pixels shifted by one, so they are read once.  The reads of row y + 1 are issued ahead of
// the MFMAs of row y and packed into fragments behind them.  D[ci][co] accumulates in registers over the unit's items, in item order, and is written to the
// unit's partial result; k_bwd_wgrad_sum adds the partial results of a (function, part) in chunk order.  Nothing is
// atomic.  The bias gradient is the same contraction with a fragment of ones in place of the input map.
struct WgArgs {
    const dynb_item* items;       // all items of the plan
    const uint8_t* arity;
    const dynb_wg_unit* units;
    const int32_t* order;         // workgroup -> unit
    const int32_t* fn_items;
    const bf16_t* feats;
    const bf16_t* slots;
    const bf16_t* sv_u;
    const bf16_t* sv_m;
    const bf16_t* sv_g;
    const bf16_t* sv_dm;
    const bf16_t* sv_dc;
    float* partial;               // [unit][3][C][C] weight gradient ([tap][co][ci]; conv1x1: tap 0 only), then [C] bias gradient
};
constexpr size_t WG_PARTIAL = size_t(3) * 128 * 128 + 128;           // floats per unit

template <int MODE>
__device__ __forceinline__ void wgrad_unit(const WgArgs& a, const dynb_wg_unit un, float* __restrict__ part_out)
{
    using namespace mf;
    constexpr int NTAP = MODE == 2 ? 1 : 3, NV = MODE == 2 ? 8 : 10, NTHR = 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int part = un.part;
    const int ar = a.arity[un.type];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, hk = lane >> 5, wi = wave & 1, wj = wave >> 1;
    constexpr uint32_t TILE_G = TILE_BYTES;                            // the gradient map's tile follows the input map's

    for (int c = tid; c < 2 * TILE_BYTES / 16; c += NTHR) reinterpret_cast<u32x4*>(lds_raw)[c] = u32x4{0u, 0u, 0u, 0u};

    f32x16 acc[NTAP][2][2], accb[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
        for (int k = 0; k < NTAP; ++k)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int cj = 0; cj < 2; ++cj) acc[k][ct][cj][i] = 0.f;
        accb[0][i] = 0.f; accb[1][i] = 0.f;
    }
    constexpr int NIT = (P * 16 + NTHR - 1) / NTHR;
    u32x4 tin[NIT], tg[NIT];
    auto load = [&](int idx) {
        const int32_t item = a.fn_items[idx];
        const dynb_item it = a.items[item];
        const size_t off = size_t(item) * (P * C);
        const bf16_t* G = (MODE == 0 ? a.sv_g : MODE == 1 ? a.sv_dm : a.sv_dc) + off;
        const bf16_t* IN;
        if (MODE == 0) IN = a.sv_m + off;
        else if (MODE == 1 && ar == 2) IN = a.sv_u + off;
        else {
            const int32_t s = (MODE == 2 && part == 1) ? it.src1 : it.src0;
            IN = s >= 0 ? a.slots + size_t(s) * (P * C) : a.feats + size_t(-1 - s) * (P * C);
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tid + i * NTHR;
            if (c < P * 16) { tin[i] = reinterpret_cast<const u32x4*>(IN)[c]; tg[i] = reinterpret_cast<const u32x4*>(G)[c]; }
        }
    };
    auto store = [&]() {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tid + i * NTHR;
            if (c < P * 16) {
                const int p = c >> 4, piece = c & 15;
                const uint32_t addr = uint32_t((p / S + 1) * ROW_BYTES + (p % S + 1) * PIX_BYTES + piece * 16);
                *reinterpret_cast<u32x4*>(lds_raw + addr) = tin[i];
                *reinterpret_cast<u32x4*>(lds_raw + TILE_G + addr) = tg[i];
            }
        }
    };
    // A wave's two channel tiles interleave: tile c of its 64 channels holds channels 2 m + c (m = MFMA row / column),
    // so that one 32-bit LDS read gives a lane its value of both tiles (a pixel's channels 2 m and 2 m + 1).
    auto rd32 = [&](uint32_t addr) -> uint32_t { return *reinterpret_cast<const uint32_t*>(lds_raw + addr); };
    // eight dwords (pixels), tile c in half c of every dword -> the 8 bf16 of tile c, one v_perm per pair of pixels
    auto frag_of = [](const uint32_t* v, int c) -> bf16x8 {
        const uint32_t sel = c ? 0x07060302u : 0x05040100u;
        auto pair = [sel](uint32_t first, uint32_t second) { return __builtin_amdgcn_perm(second, first, sel); };
        const u32x4 w = {pair(v[0], v[1]), pair(v[2], v[3]), pair(v[4], v[5]), pair(v[6], v[7])};
        return __builtin_bit_cast(bf16x8, w);
    };
    const u32x4 ones_w = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_w);
    // tile row / first tile column of this lane's 8 pixels of image row y:
    //   gradient map and conv1x1 input: row y + 1, column 1 + 8 hk;  conv3x3 input for kernel row kh: row y + kh, column 8 hk
    const uint32_t g_lane = TILE_G + uint32_t(ROW_BYTES + (1 + 8 * hk) * PIX_BYTES + (wj * 64 + 2 * m) * 2);
    const uint32_t in_lane = MODE == 2 ? uint32_t(ROW_BYTES + (1 + 8 * hk) * PIX_BYTES + (wi * 64 + 2 * m) * 2)
                                       : uint32_t(part * ROW_BYTES + (8 * hk) * PIX_BYTES + (wi * 64 + 2 * m) * 2);
    struct Raw { uint32_t g[8]; uint32_t in[NV]; };                    // one row's values as they come from LDS
    struct Row { bf16x8 gf[2]; bf16x8 inf[2][NTAP]; };                 // ... and packed into operand fragments
    // The upper lane half's last pixels do not exist (x = 14, 15) or lie beyond the tile (conv3x3 input, tile columns
    // 16, 17).  Tile column 15 is the zero border: the gradient map's x = 14 is that column already, and the lanes
    // whose pixel would lie beyond it read column 15 again, so every such value is a zero without any select.
    constexpr int ILIM = MODE == 2 ? 7 : 8;                            // first index of an input value beyond column 15
    const uint32_t g_off7 = (hk ? 6u : 7u) * PIX_BYTES;
    const uint32_t in_offa = (hk ? uint32_t(ILIM - 1) : uint32_t(ILIM)) * PIX_BYTES;
    const uint32_t in_offb = (hk ? uint32_t(ILIM - 1) : uint32_t(ILIM + 1)) * PIX_BYTES;
    const uint32_t g_lane7 = g_lane + g_off7, in_lanea = in_lane + in_offa, in_laneb = in_lane + in_offb;
    auto issue_row = [&](int y, Raw& rw) {
        const uint32_t yo = uint32_t(y * ROW_BYTES);
        const uint32_t gb = g_lane + yo, g7 = g_lane7 + yo, ib = in_lane + yo, ia = in_lanea + yo, ibb = in_laneb + yo;
#pragma unroll
        for (int i = 0; i < 7; ++i) rw.g[i] = rd32(gb + uint32_t(i * PIX_BYTES));
        rw.g[7] = rd32(g7);
#pragma unroll
        for (int i = 0; i < ILIM; ++i) rw.in[i] = rd32(ib + uint32_t(i * PIX_BYTES));
        rw.in[ILIM] = rd32(ia);
        if (ILIM + 1 < NV) rw.in[ILIM + 1 < NV ? ILIM + 1 : 0] = rd32(ibb);
    };
    auto pack_row = [&](const Raw& rw, Row& row) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            row.gf[c] = frag_of(rw.g, c);
#pragma unroll
            for (int k = 0; k < NTAP; ++k) row.inf[c][k] = frag_of(rw.in + k, c);
        }
    };
    const bool with_bias = part == 0 && wi == 0;                      // uniform over the wave
    auto mfma_row = [&](const Row& rw, auto WB) {
#pragma unroll
        for (int k = 0; k < NTAP; ++k)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int cj = 0; cj < 2; ++cj)
                    acc[k][ct][cj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rw.inf[ct][k], rw.gf[cj], acc[k][ct][cj], 0, 0, 0);
        if constexpr (decltype(WB)::value) {
#pragma unroll
            for (int cj = 0; cj < 2; ++cj) accb[cj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, rw.gf[cj], accb[cj], 0, 0, 0);
        }
    };
    // One step of the row pipeline: the LDS reads of the row after next are issued first, then the MFMAs of row `cur`
    // run with the packing of row `nxt` (whose reads were issued a step earlier) spread between them: a wave issues one
    // instruction at a time, and only what it issues while an MFMA executes is free.
    auto step = [&](int y_issue, Raw& raw_issue, const Raw& raw_pack, Row& nxt, const Row& cur, auto WB) {
        issue_row(y_issue, raw_issue);
        mfma_row(cur, WB);
        pack_row(raw_pack, nxt);
        constexpr int NMF = NTAP * 4 + (decltype(WB)::value ? 2 : 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 8 + NV, 0);                   // all reads
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);                        // (their addresses)
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, MODE == 2 ? 8 : 4, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto items = [&](auto WB) {
        load(un.begin);
        for (int idx = un.begin; idx < un.end; ++idx) {
            __syncthreads();                                          // the previous item's fragments have been read
            store();
            __syncthreads();
            if (idx + 1 < un.end) load(idx + 1);                      // arrives under this item's MFMAs
            Raw r0, r1;
            Row ra, rb;
            issue_row(0, r0);
            issue_row(1, r1);
            pack_row(r0, ra);
            __builtin_amdgcn_sched_barrier(0);
            // rows y and y + 1 per trip: r1 holds row y + 1 on entry, ra row y
#pragma unroll 1
            for (int y = 0; y < S; y += 2) {
                step(y + 2 < S ? y + 2 : y, r0, r1, rb, ra, WB);      // reads row y+2, MFMAs row y, packs row y+1
                step(y + 3 < S ? y + 3 : y, r1, r0, ra, rb, WB);      // reads row y+3, MFMAs row y+1, packs row y+2
            }
        }
    };
    if (with_bias) items(std::true_type{});
    else items(std::false_type{});
    // D[ci][co] of tiles (ct, cj): this lane holds co = wj*64 + 2 m + cj and, in elements 4 b .. 4 b + 3, the rows
    // 8 b + 4 hk + (0..3), i.e. ci = wi*64 + 2 (8 b + 4 hk + e) + ct: the two ci tiles together give 8 consecutive ci
#pragma unroll
    for (int cj = 0; cj < 2; ++cj) {
        const int co = wj * 64 + 2 * m + cj;
#pragma unroll
        for (int k = 0; k < NTAP; ++k)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int ci = wi * 64 + 16 * b + 8 * hk;
                float* dst = part_out + (size_t(k) * C + co) * C + ci;
                *reinterpret_cast<f32x4*>(dst) = f32x4{acc[k][0][cj][4 * b], acc[k][1][cj][4 * b], acc[k][0][cj][4 * b + 1], acc[k][1][cj][4 * b + 1]};
                *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[k][0][cj][4 * b + 2], acc[k][1][cj][4 * b + 2], acc[k][0][cj][4 * b + 3], acc[k][1][cj][4 * b + 3]};
            }
        if (with_bias && hk == 0) part_out[size_t(3) * C * C + co] = accb[cj][0];
    }
}

__global__ __launch_bounds__(256, 1) void k_bwd_wgrad_mfma(WgArgs a)
{
    const int32_t u = a.order[blockIdx.x];
    const dynb_wg_unit un = a.units[u];
    float* out = a.partial + size_t(u) * WG_PARTIAL;
    if (un.mode == 0) wgrad_unit<0>(a, un, out);
    else if (un.mode == 1) wgrad_unit<1>(a, un, out);
    else wgrad_unit<2>(a, un, out);
}

// dW / db of one (mode, function, part) = its units' partial results added in chunk order
struct WsArgs {
    const dynb_wg_group* groups;
    const float* partial;
    float* dw3a; float* db3a; float* dw3b; float* db3b; float* dw1; float* db1;
};

__global__ void k_bwd_wgrad_sum(WsArgs a)
{
    constexpr int C = 128;
    const dynb_wg_group g = a.groups[blockIdx.y];
    const int ntap = g.mode == 2 ? 1 : 3;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;              // float4 index inside [tap][co][ci]
    if (e < ntap * C * C / 4) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < g.n_units; ++c) {
            const f32x4 v = reinterpret_cast<const f32x4*>(a.partial + size_t(g.first_unit + c) * WG_PARTIAL)[e];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        const int ci = (e * 4) % C, co = (e * 4 / C) % C, k = e * 4 / (C * C);
        float* dst = g.mode == 2 ? a.dw1 + (size_t(g.type) * C + co) * (2 * C) + g.part * C + ci
                                 : (g.mode == 0 ? a.dw3b : a.dw3a) + ((size_t(g.type) * C + co) * 9 + g.part * 3 + k) * C + ci;
        *reinterpret_cast<f32x4*>(dst) = s;
    }
    if (g.part == 0 && blockIdx.x == 0 && threadIdx.x < C) {
        float s = 0.f;
        for (int c = 0; c < g.n_units; ++c) s += a.partial[size_t(g.first_unit + c) * WG_PARTIAL + size_t(3) * C * C + threadIdx.x];
        (g.mode == 2 ? a.db1 : g.mode == 0 ? a.db3b : a.db3a)[size_t(g.type) * C + threadIdx.x] = s;
    }
}

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
size_t elt_bytes(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

struct BwdLayout {
    size_t gy, gleaf, tmp_u, tmp_m, tmp_g, tmp_dm, tmp_du, total;
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
    // the routing tables were uploaded with the plan
    const dynb_keep_tables KT = dynb_plan_keep_tables(p);
    const char* pd = static_cast<const char*>(p->dev_buf);
    const int32_t* d_leaf_first = reinterpret_cast<const int32_t*>(pd + KT.leaf_first);
    const int32_t* d_root_item = reinterpret_cast<const int32_t*>(pd + KT.root_item);

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
            ba.gdst0 = reinterpret_cast<const int32_t*>(pd + KT.gdst0) + first;
            ba.gdst1 = reinterpret_cast<const int32_t*>(pd + KT.gdst1) + first;
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

#ifdef DYNB_BWD_FORCE_GENERIC          // development aid: the generic kernels at every shape
bool fast_shape(const dynb_shape*) { return false; }
#else
bool fast_shape(const dynb_shape* s) { return s->dtype == DYNB_BF16 && s->C == 128 && s->H == 14 && s->W == 14; }
#endif

// workspace of the MFMA path
struct BmLayout {
    size_t gy, gleaf, sv_g, sv_dm, sv_dc, pk3bT, pk3aT, pk1T;
    size_t partial, total;
};

BmLayout bm_layout(const dynb_plan* p)
{
    BmLayout L;
    const size_t chw = size_t(mf::P) * mf::C, n_items = p->items.size(), nt = size_t(p->n_types);
    const size_t n_leaf = p->leaf_first.empty() ? 0 : size_t(p->leaf_first.back());
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(std::max<size_t>(bytes, 4)); return at; };
    L.gy = take(n_items * chw * 4);
    L.gleaf = take(n_leaf * chw * 4);
    L.sv_g = take(n_items * chw * 2);
    L.sv_dm = take(n_items * chw * 2);
    L.sv_dc = take(p->has_binary ? n_items * chw * 2 : 0);
    L.pk3bT = take(nt * 9 * 128 * 128 * 2);
    L.pk3aT = take(nt * 9 * 128 * 128 * 2);
    L.pk1T = take(nt * 2 * 128 * 128 * 2);
    L.partial = take(p->wg_units.size() * WG_PARTIAL * 4);
    L.total = o;
    return L;
}

int run_backward_mfma(const dynb_plan* p, const dynb_module_weights* w, const void* feats, const void* out, const void* fwd_ws,
                      const float* dout, const dynb_module_grads* g, char* ws, hipStream_t st)
{
    static std::atomic<uint64_t> attr_set{0};                 // one bit per device
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
    if (!(attr_set.load() >> (dev & 63) & 1)) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_bwd_node_mfma<8>), hipFuncAttributeMaxDynamicSharedMemorySize, bn::LDS_BYTES),
                "hipFuncSetAttribute(k_bwd_node_mfma)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_bwd_wgrad_mfma), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * mf::TILE_BYTES),
                "hipFuncSetAttribute(k_bwd_wgrad_mfma)");
        attr_set.fetch_or(uint64_t(1) << (dev & 63));
    }
    const BmLayout L = bm_layout(p);
    const size_t chw = size_t(mf::P) * mf::C, n_items_all = p->items.size();
    const int C = mf::C, B = p->B, nt = p->n_types;
    // the routing tables, item lists and work units were uploaded with the plan
    const dynb_keep_tables KT = dynb_plan_keep_tables(p);
    const char* pd = static_cast<const char*>(p->dev_buf);
    const int32_t* d_leaf_first = reinterpret_cast<const int32_t*>(pd + KT.leaf_first);
    const int32_t* d_root_item = reinterpret_cast<const int32_t*>(pd + KT.root_item);

    // (the parameter gradients of every function are written by k_bwd_wgrad_sum, zeros included; without a
    // two-argument function in the batch there is no conv1x1 gradient to sum)
    if (!p->has_binary) {
        auto fill = [&](float* ptr, size_t n) {
            if (ptr && n) hipLaunchKernelGGL(k_bwd_fill, dim3(unsigned(std::min<size_t>((n + 255) / 256, 4096))), dim3(256), 0, st, ptr, n, 0.f);
        };
        fill(g->dw1, size_t(nt) * C * 2 * C);
        fill(g->db1, size_t(nt) * C);
    }

    // weights in fragment order, as given and transposed
    auto pack = [&](const void* src, size_t at, int ntap, int mode) {
        const size_t pieces = size_t(nt) * 4 * ntap * 512;
        hipLaunchKernelGGL(k_bwd_pack, dim3(unsigned(std::min<size_t>((pieces + 255) / 256, 4096))), dim3(256), 0, st,
                           static_cast<const bf16_t*>(src), reinterpret_cast<u32x4*>(ws + at), nt, ntap, mode);
    };
    pack(w->w3b, L.pk3bT, 9, 1);
    pack(w->w3a, L.pk3aT, 9, 1);
    if (p->has_binary) pack(w->w1, L.pk1T, 2, 3);

    float* gy = reinterpret_cast<float*>(ws + L.gy);
    const unsigned bx_map = unsigned(std::min<size_t>((chw + 255) / 256, 64));
    for (int e0 = 0; e0 < B; e0 += 32768)
        hipLaunchKernelGGL(k_bwd_seed, dim3(bx_map, unsigned(std::min(32768, B - e0))), dim3(256), 0, st, dout + size_t(e0) * chw,
                           d_root_item + e0, gy, chw);

    const char* d = static_cast<const char*>(p->dev_buf);
    const dynb_item* d_items = reinterpret_cast<const dynb_item*>(d);
    const uint8_t* d_arity = reinterpret_cast<const uint8_t*>(d + dynb_plan_arity_offset(p));
    BmArgs a;
    a.arity = d_arity;
    a.feats = static_cast<const bf16_t*>(feats); a.out = static_cast<const bf16_t*>(out); a.slots = static_cast<const bf16_t*>(fwd_ws);
    a.pk3bT = reinterpret_cast<const bf16_t*>(ws + L.pk3bT); a.pk3aT = reinterpret_cast<const bf16_t*>(ws + L.pk3aT);
    a.pk1T = reinterpret_cast<const bf16_t*>(ws + L.pk1T);
    a.gy = gy; a.gleaf = reinterpret_cast<float*>(ws + L.gleaf);
    // u and mid of every item: where the forward pass of a DYNB_PLAN_KEEP plan put them
    a.sv_m = reinterpret_cast<const bf16_t*>(static_cast<const char*>(fwd_ws) + dynb_fast_keep_offset(p));
    a.sv_u = a.sv_m + n_items_all * chw;
    a.sv_g = reinterpret_cast<bf16_t*>(ws + L.sv_g); a.sv_dm = reinterpret_cast<bf16_t*>(ws + L.sv_dm);
    a.sv_dc = reinterpret_cast<bf16_t*>(ws + L.sv_dc);
    for (size_t li = p->launches.size(); li-- > 0;) {
        const dynb_launch& l = p->launches[li];
        a.items = d_items + l.start; a.first_item = l.start; a.count = l.count;
        a.gdst0 = reinterpret_cast<const int32_t*>(pd + KT.gdst0) + l.start;
        a.gdst1 = reinterpret_cast<const int32_t*>(pd + KT.gdst1) + l.start;
        const unsigned grid = unsigned((l.count + 7) / 8 * 8);
        hipLaunchKernelGGL((k_bwd_node_mfma<8>), dim3(grid), dim3(256), bn::LDS_BYTES, st, a);
    }
    {
        WgArgs q;
        q.items = d_items; q.arity = d_arity;
        q.units = reinterpret_cast<const dynb_wg_unit*>(pd + KT.units);
        q.order = reinterpret_cast<const int32_t*>(pd + KT.order);
        q.fn_items = reinterpret_cast<const int32_t*>(pd + KT.fn_items);
        q.feats = a.feats; q.slots = a.slots;
        q.sv_u = a.sv_u; q.sv_m = a.sv_m; q.sv_g = a.sv_g; q.sv_dm = a.sv_dm; q.sv_dc = a.sv_dc;
        q.partial = reinterpret_cast<float*>(ws + L.partial);
        if (!p->wg_units.empty())
            hipLaunchKernelGGL(k_bwd_wgrad_mfma, dim3(unsigned(p->wg_units.size())), dim3(256), 2 * mf::TILE_BYTES, st, q);
        WsArgs r;
        r.groups = reinterpret_cast<const dynb_wg_group*>(pd + KT.groups);
        r.partial = q.partial;
        r.dw3a = g->dw3a; r.db3a = g->db3a; r.dw3b = g->dw3b; r.db3b = g->db3b; r.dw1 = g->dw1; r.db1 = g->db1;
        // groups without units: the sum writes their zeros
        hipLaunchKernelGGL(k_bwd_wgrad_sum, dim3(3 * 128 * 128 / 4 / 256, unsigned(p->wg_groups.size())), dim3(256), 0, st, r);
    }
    for (int e0 = 0; e0 < B; e0 += 32768)
        hipLaunchKernelGGL(k_bwd_leaves, dim3(bx_map, unsigned(std::min(32768, B - e0))), dim3(256), 0, st, a.gleaf, d_leaf_first + e0,
                           d_root_item + e0, dout + size_t(e0) * chw, g->dfeats + size_t(e0) * chw, chw);
    HIP_TRY(hipGetLastError(), "dynbatch_backward(mfma kernels)");
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
    if (fast_shape(s)) return std::max<size_t>(bm_layout(p).total, 256);
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
    if (workspace_bytes < (fast_shape(s) ? bm_layout(p).total : bwd_layout(p, s).total))
        return fail(DYNB_E_WORKSPACE, "dynbatch_backward: workspace too small");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(DYNB_E_INVAL, "dynbatch_backward: workspace not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    if (fast_shape(s)) return run_backward_mfma(p, w, feats, out, forward_workspace, dout, grads, ws, st);
    if (s->dtype == DYNB_BF16) return run_backward<bf16_t>(p, s, w, feats, out, forward_workspace, dout, grads, ws, st);
    return run_backward<float>(p, s, w, feats, out, forward_workspace, dout, grads, ws, st);
}
