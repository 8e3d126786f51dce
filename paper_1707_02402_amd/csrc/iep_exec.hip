// GPU executor of a plan: gather -> batched residual conv module -> scatter, one launch group
// per label (paper: Methods, "each pool is executed at once"; Results / IEP, "data stacking").
//
// Two kernel families with the same semantics:
//   * k_module_mfma  — bf16, C = 128, 14 x 14: one fused kernel per launch group.  A workgroup
//                      owns one or two nodes; the node's input map is gathered straight into an
//                      LDS halo tile, conv1x1 (binary functions), conv3x3, ReLU, conv3x3, residual
//                      add and ReLU all run from that tile on MFMA, and the result is scattered to
//                      the node's slot (or to the output tensor for a root).
//   * generic kernels — any C/H/W, fp32 or bf16 storage, fp32 accumulate, one thread per output
//                      element; three small kernels per launch group.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <string>

#include "device_utils.h"
#include "plan_internal.h"
#include "timing.h"

using dynb::fail;

#define HIP_TRY(expr, what)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(DYNB_E_HIP, std::string(what) + ": " + hipGetErrorString(e_));        \
    } while (0)

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

// out[example] = feats[example] for programs that are a single SCENE token
__global__ void k_copy_leaf_roots(const int32_t* examples, int n, const uint32_t* feats, uint32_t* out,
                                  size_t words_per_map)
{
    const int ex = examples[blockIdx.y];
    for (size_t w = size_t(blockIdx.x) * blockDim.x + threadIdx.x; w < words_per_map;
         w += size_t(gridDim.x) * blockDim.x)
        out[size_t(ex) * words_per_map + w] = feats[size_t(ex) * words_per_map + w];
}

// ------------------------------------------------------------------------------------------
// Fused MFMA module kernel: bf16, C = 128, 14 x 14
// ------------------------------------------------------------------------------------------
namespace mf {
constexpr int C = 128;
constexpr int S = 14;                    // spatial size
constexpr int P = S * S;                 // 196 pixels
constexpr int HALO = 16;                 // tile side with zero border
constexpr int PIX_BYTES = 272;           // 128 channels bf16 + 16 bytes pad: 17 granules of 16 bytes
// Row pitch in 16-byte granules is 16*17 + 14 = 286 = 14 (mod 16), so that the 16 consecutive
// raster pixels of one MFMA fragment (which cross a 14-pixel image row) still fall on 16 distinct
// granules mod 16, i.e. on all 64 LDS banks: pixel (y, x) sits at granule 14 y + x (mod 16).
constexpr int ROW_BYTES = HALO * PIX_BYTES + 14 * 16;  // 4576
constexpr int TILE_BYTES = HALO * ROW_BYTES;           // 73216
constexpr int MT = 13;                   // pixel tiles of 16: 208 >= 196
constexpr int CENTER = ROW_BYTES + PIX_BYTES;           // (+1,+1) from the top-left tap
constexpr int MAP_BYTES = P * C * 2;     // 50176
}  // namespace mf

// Development aid, compiled in only with -DDYNB_PHASE_CLOCKS: lane 0 of every wave stores the
// shader clock at the phase boundaries of k_module_mfma into a caller-provided device buffer.
#ifdef DYNB_PHASE_CLOCKS
__device__ long long* g_phase_clk = nullptr;      // [workgroup][wave][16]
#define PHASE(i)                                                                             \
    do {                                                                                     \
        if ((threadIdx.x & 63) == 0 && g_phase_clk)                                          \
            g_phase_clk[(size_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * 16 + (i)] = clock64(); \
    } while (0)
#else
#define PHASE(i) do {} while (0)
#endif

struct MfArgs {
    const dynb_item* items;
    int32_t count;
    int32_t any_binary;
    const uint8_t* arity;     // device [n_types]
    const bf16_t* feats;
    bf16_t* out;
    bf16_t* slots;
    const bf16_t* w1;
    const float* b1;
    const bf16_t* w3a;
    const float* b3a;
    const bf16_t* w3b;
    const float* b3b;
};

__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t addr)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    return *reinterpret_cast<const bf16x8*>(lds_raw + addr);
}

// K-loop shared by the 3x3 convolutions (9 taps x 4 chunks of 32 input channels) and by each half
// of the 1x1 convolution (centre tap only, 4 chunks):
//     acc[mt][nt] += W[co, tap, chunk] * X[pixel + tap, chunk]
// Software pipelined by hand.  The 13 activation fragments of a step live in one of two register
// sets (xa / xb): while the MFMAs of a step read one set, the LDS reads of the next step fill the
// other.  Weight fragments sit in a ring of four (indexed by the chunk number) and are fetched from
// global memory two steps ahead.  The tap loop stays rolled: four steps per iteration return every
// ring to the same phase at the back edge.
template <int NT, bool CENTER_ONLY>
__device__ __forceinline__ void kloop_mfma(f32x4 (&acc)[mf::MT][NT], const uint32_t (&xaddr)[mf::MT],
                                           const bf16_t* (&wrow)[NT])
{
    // wrow[nt] points at W[co = n0 + nt*16 + lane%16][tap 0][ci = (lane/16)*8]
    constexpr int NTAP = CENTER_ONLY ? 1 : 9;
    bf16x8 xa[mf::MT], xb[mf::MT], wf[4][NT];
    auto tap_off = [](int tap) -> uint32_t {
        return CENTER_ONLY ? uint32_t(mf::CENTER) : uint32_t((tap / 3) * mf::ROW_BYTES + (tap % 3) * mf::PIX_BYTES);
    };
    auto load_x = [&](bf16x8 (&x)[mf::MT], uint32_t off) {
#pragma unroll
        for (int mt = 0; mt < mf::MT; ++mt) x[mt] = lds_read_frag(xaddr[mt] + off);
    };
    auto load_w = [&](bf16x8 (&w)[NT], int off) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) w[nt] = *reinterpret_cast<const bf16x8*>(wrow[nt] + off);
    };
    // One K-step: the MFMAs of pixel tile mt read xc[mt]; the LDS read that fills xn[mt] for the next
    // step is issued right before them, so LDS traffic is spread evenly under the MFMAs instead of
    // arriving as a burst of 13 reads.  The fences keep the scheduler from regrouping the pairs.
    auto step = [&](const bf16x8 (&xc)[mf::MT], bf16x8 (&xn)[mf::MT], uint32_t noff, const bf16x8 (&w)[NT]) {
#pragma unroll
        for (int mt = 0; mt < mf::MT; ++mt) {
            xn[mt] = lds_read_frag(xaddr[mt] + noff);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nt], xc[mt], acc[mt][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    load_w(wf[0], 0);
    load_w(wf[1], 32);
    load_x(xa, tap_off(0));
#pragma unroll 1
    for (int tap = 0; tap < NTAP; ++tap) {
        const int ntap = tap + 1 < NTAP ? tap + 1 : tap;      // the last prefetch re-reads valid data
        const uint32_t xo = tap_off(tap), nxo = tap_off(ntap);
        const int wo = tap * mf::C, nwo = ntap * mf::C;
        load_w(wf[2], wo + 64);
        __builtin_amdgcn_sched_barrier(0);
        step(xa, xb, xo + 64, wf[0]);
        load_w(wf[3], wo + 96);
        __builtin_amdgcn_sched_barrier(0);
        step(xb, xa, xo + 128, wf[1]);
        load_w(wf[0], nwo);
        __builtin_amdgcn_sched_barrier(0);
        step(xa, xb, xo + 192, wf[2]);
        load_w(wf[1], nwo + 32);
        __builtin_amdgcn_sched_barrier(0);
        step(xb, xa, nxo, wf[3]);
    }
}

template <int NT>
__device__ __forceinline__ void conv3x3_mfma(f32x4 (&acc)[mf::MT][NT], const uint32_t (&xaddr)[mf::MT],
                                             const bf16_t* (&wrow)[NT])
{
    kloop_mfma<NT, false>(acc, xaddr, wrow);
}

// half of the 1x1 convolution over the concatenated arguments: 4 K-steps over the map now in LDS
template <int NT>
__device__ __forceinline__ void conv1x1_half_mfma(f32x4 (&acc)[mf::MT][NT], const uint32_t (&xaddr)[mf::MT],
                                                  const bf16_t* (&wrow)[NT])
{
    kloop_mfma<NT, true>(acc, xaddr, wrow);
}

// NPW = nodes per workgroup (1 or 2).  256 threads = 4 waves; a node is shared by 4/NPW waves,
// each owning 128/(4/NPW) output channels for all 196 pixels.
template <int NPW>
__global__ __launch_bounds__(256) void k_module_mfma(MfArgs a)
{
    using namespace mf;
    constexpr int WPN = 4 / NPW;          // waves per node
    constexpr int NT = 8 / WPN;           // 16-channel tiles per wave
    constexpr int NTHR = 64 * WPN;        // threads that stage one node
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

    // Workgroup -> position in the launch group.  Consecutive workgroup ids land on different
    // XCDs; give every XCD one contiguous run of items (items are sorted by function id) so that
    // a function's weights stay in as few L2s as possible.
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int first = logical * NPW;
    if (first >= a.count) return;

    PHASE(0);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int node_local = wave / WPN;
    const bool active = first + node_local < a.count;                 // wave-uniform
    const dynb_item it = a.items[active ? first + node_local : first];
    const bool binary = active && a.arity[it.type] == 2;
    const uint32_t tile = uint32_t(node_local) * TILE_BYTES;
    const int r = lane & 15, g = lane >> 4;
    const int n0 = (wave % WPN) * NT * 16;

    // ---- gather: zero border once, then the argument map into the centre of the halo tile
    const int tl = tid % NTHR;
    // all global loads of the map are issued before the first LDS write, so one memory latency is paid
    auto stage = [&](const bf16_t* src) {
        constexpr int NIT = (P * 16 + NTHR - 1) / NTHR;
        const u32x4* s4 = reinterpret_cast<const u32x4*>(src);
        u32x4 tmp[NIT];
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tl + i * NTHR;
            if (c < P * 16) tmp[i] = s4[c];
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = tl + i * NTHR;
            if (c < P * 16) {
                const int p = c >> 4, part = c & 15;
                const uint32_t addr = tile + uint32_t((p / S + 1) * ROW_BYTES + (p % S + 1) * PIX_BYTES + part * 16);
                *reinterpret_cast<u32x4*>(lds_raw + addr) = tmp[i];
            }
        }
    };
    if (active) {
        for (int c = tl; c < 60 * 16; c += NTHR) {
            const int q = c >> 4, part = c & 15;
            int row, col;
            if (q < 16) { row = 0; col = q; }
            else if (q < 32) { row = HALO - 1; col = q - 16; }
            else { row = 1 + ((q - 32) >> 1); col = ((q - 32) & 1) ? HALO - 1 : 0; }
            *reinterpret_cast<u32x4*>(lds_raw + tile + uint32_t(row * ROW_BYTES + col * PIX_BYTES + part * 16)) =
                u32x4{0u, 0u, 0u, 0u};
        }
        stage(it.src0 >= 0 ? a.slots + size_t(it.src0) * (P * C) : a.feats + size_t(-1 - it.src0) * (P * C));
    }

    // per-lane LDS addresses: top-left tap of the pixel this lane feeds to the MFMA B operand
    uint32_t xaddr[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int p = min(mt * 16 + r, P - 1);
        xaddr[mt] = tile + uint32_t((p / S) * ROW_BYTES + (p % S) * PIX_BYTES + g * 16);
    }
    const int cbase = n0 + g * 4;          // first of this lane's 4 output channels inside tile nt: + nt*16
    f32x4 acc[MT][NT];

    auto init_bias = [&](const float* b) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (b) v = *reinterpret_cast<const f32x4*>(b + size_t(it.type) * C + cbase + nt * 16);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = v;
        }
    };
    // ReLU(acc) -> bf16 -> centre of the halo tile (in place)
    auto write_tile = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt * 16 + r < P) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const uint32_t addr = xaddr[mt] - uint32_t(g * 16) + CENTER + uint32_t((cbase + nt * 16) * 2);
                    const f32x4 v = acc[mt][nt];
                    u32x2 pk;
                    pk.x = relu_bf16x2(pack_bf16x2(v.x, v.y));
                    pk.y = relu_bf16x2(pack_bf16x2(v.z, v.w));
                    *reinterpret_cast<u32x2*>(lds_raw + addr) = pk;
                }
            }
        }
    };

    PHASE(1);
    __syncthreads();
    PHASE(2);

    // ---- binary functions: u = ReLU(conv1x1(concat(arg0, arg1)) + b1), built in the same tile
    if (a.any_binary) {                                   // uniform over the launch group
        const bf16_t* w1row[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            w1row[nt] = a.w1 + (size_t(it.type) * C + n0 + nt * 16 + r) * (2 * C) + g * 8;
        if (binary) {
            init_bias(a.b1);
            conv1x1_half_mfma<NT>(acc, xaddr, w1row);
        }
        __syncthreads();
        if (binary) stage(it.src1 >= 0 ? a.slots + size_t(it.src1) * (P * C) : a.feats + size_t(-1 - it.src1) * (P * C));
        __syncthreads();
        if (binary) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) w1row[nt] += C;
            conv1x1_half_mfma<NT>(acc, xaddr, w1row);
        }
        __syncthreads();
        if (binary) write_tile();
        __syncthreads();
    }

    // ---- first conv3x3 + ReLU, result replaces the tile; the old centre values become the residual
    PHASE(3);
    const bf16_t* wrow[NT];
    if (active) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            wrow[nt] = a.w3a + (size_t(it.type) * C + n0 + nt * 16 + r) * (9 * C) + g * 8;
        init_bias(a.b3a);
        conv3x3_mfma<NT>(acc, xaddr, wrow);
    }
    PHASE(4);
    __syncthreads();
    PHASE(5);
    if (active) {
        f32x4 bias2[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            bias2[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (a.b3b) bias2[nt] = *reinterpret_cast<const f32x4*>(a.b3b + size_t(it.type) * C + cbase + nt * 16);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt * 16 + r < P) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const uint32_t addr = xaddr[mt] - uint32_t(g * 16) + CENTER + uint32_t((cbase + nt * 16) * 2);
                    const u32x2 res = *reinterpret_cast<const u32x2*>(lds_raw + addr);
                    const f32x4 v = acc[mt][nt];
                    u32x2 pk;
                    pk.x = relu_bf16x2(pack_bf16x2(v.x, v.y));
                    pk.y = relu_bf16x2(pack_bf16x2(v.z, v.w));
                    *reinterpret_cast<u32x2*>(lds_raw + addr) = pk;
                    f32x4 nv;
                    nv.x = __uint_as_float(res.x << 16) + bias2[nt].x;
                    nv.y = __uint_as_float(res.x & 0xffff0000u) + bias2[nt].y;
                    nv.z = __uint_as_float(res.y << 16) + bias2[nt].z;
                    nv.w = __uint_as_float(res.y & 0xffff0000u) + bias2[nt].w;
                    acc[mt][nt] = nv;
                }
            }
        }
    }
    PHASE(6);
    __syncthreads();
    PHASE(7);

    // ---- second conv3x3 on top of (residual + bias), ReLU, scatter
    if (active) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            wrow[nt] = a.w3b + (size_t(it.type) * C + n0 + nt * 16 + r) * (9 * C) + g * 8;
        conv3x3_mfma<NT>(acc, xaddr, wrow);
        PHASE(8);
        bf16_t* dst = it.dst >= 0 ? a.slots + size_t(it.dst) * (P * C) : a.out + size_t(-1 - it.dst) * (P * C);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int p = mt * 16 + r;
            if (p < P) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const f32x4 v = acc[mt][nt];
                    u32x2 pk;
                    pk.x = relu_bf16x2(pack_bf16x2(v.x, v.y));
                    pk.y = relu_bf16x2(pack_bf16x2(v.z, v.w));
                    *reinterpret_cast<u32x2*>(dst + size_t(p) * C + cbase + nt * 16) = pk;
                }
            }
        }
    }
    PHASE(9);
}

size_t elt_bytes(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

bool fast_shape(const dynb_shape* s) { return s->dtype == DYNB_BF16 && s->C == 128 && s->H == 14 && s->W == 14; }

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

}  // namespace

#ifdef DYNB_PHASE_CLOCKS
extern "C" int dynb_debug_phase_clocks(void* device_buf)
{
    long long* p = static_cast<long long*>(device_buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_phase_clk), &p, sizeof(p)) == hipSuccess ? DYNB_OK : DYNB_E_HIP;
}
#endif

// Device buffer layout of an uploaded plan: items | leaf-root example ids | arity table
static size_t plan_items_bytes(const dynb_plan* p) { return align256(p->items.size() * sizeof(dynb_item)); }
static size_t plan_leaf_bytes(const dynb_plan* p) { return align256(p->leaf_roots.size() * sizeof(int32_t)); }

extern "C" size_t dynbatch_plan_device_bytes(const dynb_plan* p)
{
    if (!p) return 0;
    return plan_items_bytes(p) + plan_leaf_bytes(p) + align256(p->arity.size()) + 256;
}

extern "C" int dynbatch_plan_upload(dynb_plan* p, void* dev_buf, size_t bytes, void* stream)
{
    if (!p || !dev_buf) return fail(DYNB_E_INVAL, "dynbatch_plan_upload: NULL argument");
    if (bytes < dynbatch_plan_device_bytes(p)) return fail(DYNB_E_WORKSPACE, "dynbatch_plan_upload: buffer too small");
    if (reinterpret_cast<uintptr_t>(dev_buf) & 15) return fail(DYNB_E_INVAL, "dynbatch_plan_upload: buffer not 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* d = static_cast<char*>(dev_buf);
    if (!p->items.empty())
        HIP_TRY(hipMemcpyAsync(d, p->items.data(), p->items.size() * sizeof(dynb_item), hipMemcpyHostToDevice, st),
                "dynbatch_plan_upload(items)");
    if (!p->leaf_roots.empty())
        HIP_TRY(hipMemcpyAsync(d + plan_items_bytes(p), p->leaf_roots.data(), p->leaf_roots.size() * sizeof(int32_t),
                               hipMemcpyHostToDevice, st),
                "dynbatch_plan_upload(leaf roots)");
    HIP_TRY(hipMemcpyAsync(d + plan_items_bytes(p) + plan_leaf_bytes(p), p->arity.data(), p->arity.size(),
                           hipMemcpyHostToDevice, st),
            "dynbatch_plan_upload(arity)");
    p->dev_buf = dev_buf;
    p->dev_bytes = bytes;
    return DYNB_OK;
}

extern "C" size_t dynbatch_workspace_bytes(const dynb_plan* p, const dynb_shape* s)
{
    if (!p || !s || s->C <= 0 || s->H <= 0 || s->W <= 0) return 0;
    if (s->dtype != DYNB_F32 && s->dtype != DYNB_BF16) return 0;
    const size_t map = size_t(s->C) * s->H * s->W * elt_bytes(s->dtype);    // slots are packed
    size_t n = size_t(p->n_slots);
    if (!fast_shape(s)) n += 2 * size_t(p->max_launch);                       // u and mid of one launch group
    return std::max<size_t>(align256(n * map), 256);
}

template <typename T>
static int run_generic(const dynb_plan* p, const dynb_shape* s, const dynb_module_weights* w, const void* feats,
                       void* out, char* ws, hipStream_t st)
{
    const size_t chw = size_t(s->C) * s->H * s->W;
    const size_t map = chw * sizeof(T);
    const char* d = static_cast<const char*>(p->dev_buf);
    GenArgs a;
    a.arity = reinterpret_cast<const uint8_t*>(d + plan_items_bytes(p) + plan_leaf_bytes(p));
    a.feats = feats; a.out = out; a.slots = ws;
    a.tmp_u = ws + size_t(p->n_slots) * map;
    a.tmp_m = ws + (size_t(p->n_slots) + p->max_launch) * map;
    a.w1 = w->w1; a.b1 = w->b1; a.w3a = w->w3a; a.b3a = w->b3a; a.w3b = w->w3b; a.b3b = w->b3b;
    a.C = s->C; a.H = s->H; a.W = s->W;
    const unsigned bx = unsigned((chw + 255) / 256);
    const bool timed = dynb::timing_on();
    for (const dynb_launch& l : p->launches) {
        a.items = reinterpret_cast<const dynb_item*>(d) + l.start;
        a.count = l.count;
        bool any_binary = false;
        for (int i = 0; i < l.count; ++i) any_binary |= (p->arity[p->items[l.start + i].type] == 2);
        // grid.y is limited to 65535: split very wide launch groups
        for (int off = 0; off < l.count; off += 32768) {
            GenArgs b = a;
            b.items = a.items + off;
            b.count = std::min(32768, l.count - off);
            b.tmp_u = static_cast<char*>(a.tmp_u) + size_t(off) * map;
            b.tmp_m = static_cast<char*>(a.tmp_m) + size_t(off) * map;
            dim3 grid(bx, unsigned(b.count));
            if (any_binary) hipLaunchKernelGGL((k_gen_join<T>), grid, dim3(256), 0, st, b);
            hipLaunchKernelGGL((k_gen_conv<T, false>), grid, dim3(256), 0, st, b);
            hipLaunchKernelGGL((k_gen_conv<T, true>), grid, dim3(256), 0, st, b);
        }
        if (timed) dynb::timing_mark(st, int32_t(&l - p->launches.data()), l.count);
    }
    HIP_TRY(hipGetLastError(), "dynbatch_execute(generic kernels)");
    return DYNB_OK;
}

static int run_mfma(const dynb_plan* p, const dynb_module_weights* w, const void* feats, void* out, char* ws,
                    hipStream_t st)
{
    static std::atomic<uint64_t> attr_set{0};                 // one bit per device
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
    if (!(attr_set.load() >> (dev & 63) & 1)) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<1>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 2 * mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<2>)");
        attr_set.fetch_or(uint64_t(1) << (dev & 63));
    }
    const char* d = static_cast<const char*>(p->dev_buf);
    MfArgs a;
    a.arity = reinterpret_cast<const uint8_t*>(d + plan_items_bytes(p) + plan_leaf_bytes(p));
    a.feats = static_cast<const bf16_t*>(feats);
    a.out = static_cast<bf16_t*>(out);
    a.slots = reinterpret_cast<bf16_t*>(ws);
    a.w1 = static_cast<const bf16_t*>(w->w1); a.b1 = w->b1;
    a.w3a = static_cast<const bf16_t*>(w->w3a); a.b3a = w->b3a;
    a.w3b = static_cast<const bf16_t*>(w->w3b); a.b3b = w->b3b;
    const bool timed = dynb::timing_on();
    for (const dynb_launch& l : p->launches) {
        a.items = reinterpret_cast<const dynb_item*>(d) + l.start;
        a.count = l.count;
        a.any_binary = 0;
        for (int i = 0; i < l.count; ++i) a.any_binary |= (p->arity[p->items[l.start + i].type] == 2);
        // two nodes per workgroup once the launch group has more nodes than the chip has CUs twice over
        const int npw = (l.count > 512) ? 2 : 1;
        const int nwg = (l.count + npw - 1) / npw;
        const unsigned grid = unsigned((nwg + 7) / 8 * 8);
        if (npw == 1)
            hipLaunchKernelGGL((k_module_mfma<1>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
        else
            hipLaunchKernelGGL((k_module_mfma<2>), dim3(grid), dim3(256), 2 * mf::TILE_BYTES, st, a);
        if (timed) dynb::timing_mark(st, int32_t(&l - p->launches.data()), l.count);
    }
    HIP_TRY(hipGetLastError(), "dynbatch_execute(mfma kernels)");
    return DYNB_OK;
}

extern "C" int dynbatch_execute(const dynb_plan* p, const dynb_shape* s, const dynb_module_weights* w,
                                const void* feats, void* out, void* workspace, size_t workspace_bytes,
                                void* stream)
{
    if (!p || !s || !w || !feats || !out || !workspace) return fail(DYNB_E_INVAL, "dynbatch_execute: NULL argument");
    if (s->C <= 0 || s->H <= 0 || s->W <= 0) return fail(DYNB_E_INVAL, "dynbatch_execute: C, H, W must be positive");
    if (s->dtype != DYNB_F32 && s->dtype != DYNB_BF16) return fail(DYNB_E_UNSUPPORTED, "dynbatch_execute: unknown dtype");
    if (!w->w3a || !w->w3b) return fail(DYNB_E_INVAL, "dynbatch_execute: conv3x3 weights missing");
    if (p->has_binary && !w->w1) return fail(DYNB_E_UNSUPPORTED, "dynbatch_execute: binary functions need w1");
    if (!p->dev_buf) return fail(DYNB_E_WORKSPACE, "dynbatch_execute: plan not uploaded");
    if (workspace_bytes < dynbatch_workspace_bytes(p, s)) return fail(DYNB_E_WORKSPACE, "dynbatch_execute: workspace too small");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(DYNB_E_INVAL, "dynbatch_execute: workspace not 256-byte aligned");
    if (size_t(s->C) * s->H * s->W >= (size_t(1) << 31)) return fail(DYNB_E_UNSUPPORTED, "dynbatch_execute: map too large");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);

    if (dynb::timing_on()) dynb::timing_begin(st);
    if (!p->leaf_roots.empty()) {
        const size_t words = size_t(s->C) * s->H * s->W * elt_bytes(s->dtype) / 4;
        if ((size_t(s->C) * s->H * s->W * elt_bytes(s->dtype)) % 4) return fail(DYNB_E_UNSUPPORTED, "dynbatch_execute: odd-sized bf16 map");
        const int32_t* ex = reinterpret_cast<const int32_t*>(static_cast<const char*>(p->dev_buf) + plan_items_bytes(p));
        for (size_t off = 0; off < p->leaf_roots.size(); off += 32768) {
            const unsigned n = unsigned(std::min<size_t>(32768, p->leaf_roots.size() - off));
            dim3 grid(unsigned(std::min<size_t>((words + 255) / 256, 64)), n);
            hipLaunchKernelGGL(k_copy_leaf_roots, grid, dim3(256), 0, st, ex + off, int(n),
                               static_cast<const uint32_t*>(feats), static_cast<uint32_t*>(out), words);
        }
    }
    if (p->items.empty()) {
        HIP_TRY(hipGetLastError(), "dynbatch_execute(copy)");
        return DYNB_OK;
    }
    if (fast_shape(s)) return run_mfma(p, w, feats, out, ws, st);
    if (s->dtype == DYNB_BF16) return run_generic<bf16_t>(p, s, w, feats, out, ws, st);
    return run_generic<float>(p, s, w, feats, out, ws, st);
}
