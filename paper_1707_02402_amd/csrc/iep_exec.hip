// GPU executor of a plan: gather -> batched residual conv module -> scatter, one launch group
// per label (paper: Methods / Improved topological sort, a pool is executed as one batch; Results / IEP, data stacking).
//
// Two kernel families with the same semantics:
//   * k_module_mfma  — bf16, C = 128, 14 x 14: one fused kernel per launch group.  A workgroup
//                      owns a node or half a node; the node's input map is gathered straight into an
//                      LDS halo tile, conv1x1 (binary functions), conv3x3, ReLU, conv3x3, residual
//                      add and ReLU all run from that tile on MFMA, and the result is scattered to
//                      the node's slot (or to the output tensor for a root).
//   * generic kernels — any C/H/W, fp32 or bf16 storage, fp32 accumulate, one thread per output
//                      element; three small kernels per launch group.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <string>

#include "device_utils.h"
#include "iep_generic.h"
#include "iep_mfma.h"
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

// out[example] = feats[example] for programs that are a single SCENE token
__global__ void k_copy_leaf_roots(const int32_t* examples, int n, const uint32_t* feats, uint32_t* out,
                                  size_t words_per_map)
{
    if (int(blockIdx.y) >= n) return;
    const int ex = examples[blockIdx.y];
    for (size_t w = size_t(blockIdx.x) * blockDim.x + threadIdx.x; w < words_per_map;
         w += size_t(gridDim.x) * blockDim.x)
        out[size_t(ex) * words_per_map + w] = feats[size_t(ex) * words_per_map + w];
}

// ------------------------------------------------------------------------------------------
// Fused MFMA module kernel: bf16, C = 128, 14 x 14
// ------------------------------------------------------------------------------------------
// Development aid, compiled in only with -DDYNB_PHASE_CLOCKS: lane 0 of every wave stores the
// shader clock at the phase boundaries of k_module_mfma into a caller-provided device buffer.
#ifdef DYNB_PHASE_CLOCKS
__device__ long long* g_phase_clk = nullptr;      // [workgroup][wave][16]
#define PHASE(i)                                                                             \
    do {                                                                                     \
        if ((threadIdx.x & 63) == 0 && g_phase_clk)                                          \
            g_phase_clk[(size_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * 16 + (i)] = clock64(); \
        if ((threadIdx.x & 63) == 0 && g_phase_clk && ((i) == 0 || (i) == 9))                 \
            g_phase_clk[(size_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * 16 + 10 + ((i) != 0)] = wall_clock64(); \
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
    // plans that keep what the backward pass needs: u of two-argument functions and mid, one map per item
    int32_t first_item;       // index of items[0] in the plan
    bf16_t* keep_u;           // [n_items][P*C]
    bf16_t* keep_m;
};


// dst[function][tile][tap][j][lane][i] = src[function][co = tile*32 + rho(lane%32)][tap][ci = (lane/32)*64 + j*8 + i]
// one thread per 16-byte piece; ntap = 9 for a conv3x3, 2 for the two halves of the conv1x1 over 2C inputs.
// rho permutes the channels inside a tile: MFMA output row m = 8b + 4h + c (accumulator element 4b + c
// of lane half h) is given channel 16h + 4b + c, so that the 16 accumulator elements of a lane are 16
// consecutive channels and leave the kernel as two 16-byte stores.
__global__ void k_pack_weights(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int n_types, int ntap)
{
    const size_t total = size_t(n_types) * 4 * ntap * 8 * 64;
    for (size_t q = size_t(blockIdx.x) * blockDim.x + threadIdx.x; q < total; q += size_t(gridDim.x) * blockDim.x) {
        const int lane = int(q & 63), j = int((q >> 6) & 7);
        const size_t rest = q >> 9;
        const int tap = int(rest % ntap), tile = int((rest / ntap) & 3);
        const size_t type = rest / (size_t(ntap) * 4);
        const int m = lane & 31;
        const int co = tile * 32 + ((m >> 2) & 1) * 16 + (m >> 3) * 4 + (m & 3), ci0 = (lane >> 5) * 64 + j * 8;
        dst[q] = src[(((type * 128 + co) * ntap + tap) * 128 + ci0) >> 3];
    }
}

// WM selects how a node is spread over workgroups.
//   WM = 2: one node per workgroup: wave w owns channel tile w (32 channels) and all 7 pixel tiles.
//   WM = 3: half a node per workgroup: output rows 0..6 or 7..13.  The workgroup convolves an 8-row window (rows
//           0..7 or 6..13: the second conv needs one row of the first conv's output beyond its own rows), i.e. 112
//           pixels = 4 pixel tiles; wave w owns channel tile w of all four.  Two CUs share a node, which halves the
//           latency of narrow launch groups at the price of 8/7 of the MFMA work.
//   WM = 4: the layout of WM = 2 inside at most 256 registers (two sets of activation fragments instead of four),
//           so that two workgroups share a CU and one's staging, swap and epilogue run under the other's MFMAs.
// WM = 2 and 3 own a CU (up to 512 registers per lane) and, unless ALLOW_DEEP is off, keep a weight ring of 24
// steps that is filled before the argument map is staged.
// One workgroup's share of a launch group: position `logical` (a node, half a node or a pair of nodes,
// depending on the layout) of the items a.items[0 .. a.count).
// KEEP: u (two-argument functions) and mid are also written to a.keep_u / a.keep_m, as they enter the LDS tile.
template <int WMODE, bool ALLOW_DEEP = true, bool KEEP = false>
__device__ __forceinline__ void module_body(const MfArgs& a, const int logical)
{
    using namespace mf;
    static_assert(WMODE == 2 || WMODE == 3 || WMODE == 4, "layouts");
    constexpr int WM = (WMODE == 4) ? 2 : WMODE;
    constexpr int NPW = 1;                    // nodes per workgroup
    constexpr int WPN = 4;                    // waves per node
    constexpr int NT = 1;                     // channel tiles per wave
    constexpr bool HALF = (WM == 3);
    constexpr int MTW = HALF ? 4 : MT7;       // pixel tiles per wave: all of the node's (or of the half node's window)
    constexpr int NTHR = 64 * WPN;            // threads that stage one node
    constexpr bool DEEP = ALLOW_DEEP && (WMODE == 2 || WMODE == 3);
    constexpr int RW = DEEP ? 24 : 8;         // weight ring depth in K-steps
    constexpr int XS = (WMODE == 4) ? 2 : 4;  // register sets of activation fragments (look-ahead of XS / 2 steps)
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

    const int first = HALF ? (logical >> 1) : logical * NPW;
    if (first >= a.count) return;
    // pixel window of this workgroup: image rows [wrow0, wrow0 + wrows); output rows [orow0, orow1)
    const int wrow0 = HALF ? (logical & 1) * 6 : 0;
    constexpr int wrows = HALF ? 8 : S;
    constexpr int NPIX = wrows * S;           // 196 or 112
    const int orow0 = HALF ? (logical & 1) * 7 : 0, orow1 = HALF ? orow0 + 7 : S;

    PHASE(0);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int node_local = wave / WPN, wi = wave % WPN;
    const bool active = first + node_local < a.count;                 // wave-uniform
    const dynb_item it = a.items[active ? first + node_local : first];
    const bool binary = active && a.arity[it.type] == 2;
    const uint32_t tile = uint32_t(node_local) * TILE_BYTES;
    const int r = lane & 31, h = lane >> 5;
    const int n0 = wi * 32 * NT;              // first output channel of this wave

    // packed weights of this wave's channel tiles: fragment (tap, j) of a conv follows at (tap*8 + j) * FRAG
    const bf16_t* wrow_a[NT];
    const bf16_t* wrow_b[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const size_t frag0 = (size_t(it.type) * 4 + (n0 >> 5) + nt) * 9 * 8;
        wrow_a[nt] = a.w3a + frag0 * FRAG + lane * 8;
        wrow_b[nt] = a.w3b + frag0 * FRAG + lane * 8;
    }
    bf16x8 ring[RW][NT];

    // ---- gather: zero border once, then the argument map into the centre of the halo tile;
    // all global loads of the map are issued before the first LDS write, so one memory latency is paid
    const int tl = tid % NTHR;
    // rows of the argument map that the window's 3x3 taps can touch
    const int srow0 = wrow0 > 0 ? wrow0 - 1 : 0;
    const int srow1 = wrow0 + wrows + 1 < S ? wrow0 + wrows + 1 : S;
    constexpr int MAXPIECES = (HALF ? 9 : S) * S * 16;
    constexpr int NIT = (MAXPIECES + NTHR - 1) / NTHR;
    const int c_lo = srow0 * S * 16, c_hi = srow1 * S * 16;
    u32x4 tmp[NIT];
    auto stage_load = [&](const bf16_t* src) {
        const u32x4* s4 = reinterpret_cast<const u32x4*>(src);
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = c_lo + tl + i * NTHR;
            if (c < c_hi) tmp[i] = s4[c];
        }
    };
    auto stage_store = [&]() {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = c_lo + tl + i * NTHR;
            if (c < c_hi) {
                const int p = c >> 4, part = c & 15;
                const uint32_t addr = tile + uint32_t((p / S + 1) * ROW_BYTES + (p % S + 1) * PIX_BYTES + part * 16);
                *reinterpret_cast<u32x4*>(lds_raw + addr) = tmp[i];
            }
        }
    };
    auto stage = [&](const bf16_t* src) { stage_load(src); stage_store(); };
    // Loads return in the order they were issued: the argument map (needed first) goes ahead of the weight ring,
    // whose fragments then arrive while the map is written to the tile.
    if (active) stage_load(it.src0 >= 0 ? a.slots + size_t(it.src0) * (P * C) : a.feats + size_t(-1 - it.src0) * (P * C));
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DEEP)
        if (!a.any_binary) ring_fill<NT, RW>(ring, wrow_a);
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
        stage_store();
    }

    // per-lane LDS addresses: top-left tap of the pixel this lane feeds to the MFMA B operand,
    // already advanced to this lane half's 64-channel run
    uint32_t xaddr[MTW];
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        const int p = wrow0 * S + min(t * 32 + r, NPIX - 1);
        xaddr[t] = tile + uint32_t((p / S) * ROW_BYTES + (p % S) * PIX_BYTES + h * 128);
    }
    // this lane's 16 accumulator elements of channel tile nt are channels n0 + nt*32 + 16*h + (0..15)
    // (the packed weights carry the matching row permutation)
    auto chan = [&](int nt) -> int { return n0 + nt * 32 + 16 * h; };
    f32x16 acc[MTW][NT];

    auto init_bias = [&](const float* bias) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (bias) v = *reinterpret_cast<const f32x4*>(bias + size_t(it.type) * C + chan(nt) + b * 4);
#pragma unroll
                for (int t = 0; t < MTW; ++t) {
                    acc[t][nt][4 * b + 0] = v.x; acc[t][nt][4 * b + 1] = v.y;
                    acc[t][nt][4 * b + 2] = v.z; acc[t][nt][4 * b + 3] = v.w;
                }
            }
    };
    // byte address of this lane's centre pixel of tile t (channel 0)
    auto centre = [&](int t) -> uint32_t { return xaddr[t] - uint32_t(h * 128) + CENTER; };
    // ReLU(acc[t][nt][8q .. 8q+7]) as 8 packed bf16 (q = 0, 1)
    auto packed = [&](int t, int nt, int q) -> u32x4 {
        u32x4 pk;
        pk.x = relu_bf16x2(pack_bf16x2(acc[t][nt][8 * q + 0], acc[t][nt][8 * q + 1]));
        pk.y = relu_bf16x2(pack_bf16x2(acc[t][nt][8 * q + 2], acc[t][nt][8 * q + 3]));
        pk.z = relu_bf16x2(pack_bf16x2(acc[t][nt][8 * q + 4], acc[t][nt][8 * q + 5]));
        pk.w = relu_bf16x2(pack_bf16x2(acc[t][nt][8 * q + 6], acc[t][nt][8 * q + 7]));
        return pk;
    };

    PHASE(1);
    __syncthreads();
    PHASE(2);

    // ---- binary functions: u = ReLU(conv1x1(concat(arg0, arg1)) + b1), built in the same tile.
    // The first conv3x3 reads u one row beyond the window, so in half-node mode the 1x1 runs on its
    // own 9-row window (rows 0..8 or 5..13: 126 pixels, still 4 tiles).
    if (a.any_binary) {                                   // uniform over the launch group
        const int urow0 = HALF ? (wrow0 > 0 ? wrow0 - 1 : 0) : 0;
        constexpr int UPIX = HALF ? 9 * S : P;
        uint32_t uaddr[MTW];
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            const int p = urow0 * S + min(t * 32 + r, UPIX - 1);
            uaddr[t] = tile + uint32_t((p / S) * ROW_BYTES + (p % S) * PIX_BYTES + h * 128);
        }
        const bf16_t* w1row[NT];                          // first half of the 1x1 weights (argument 0), then the second
        const bf16_t* w1row2[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            w1row[nt] = a.w1 + ((size_t(it.type) * 4 + (n0 >> 5) + nt) * 2 * 8) * FRAG + lane * 8;
            w1row2[nt] = w1row[nt] + 8 * FRAG;
        }
        // the second half's fragments are fetched under the first half's loop and wait in the ring while the second
        // argument is staged
        bf16x8 ring1[8][NT];
        if (binary) {
            ring_fill<NT, 8>(ring1, w1row);
            init_bias(a.b1);
            kloop<MTW, NT, 8, XS, true>(acc, uaddr, ring1, w1row, w1row2);
        }
        __syncthreads();
        if (binary) stage(it.src1 >= 0 ? a.slots + size_t(it.src1) * (P * C) : a.feats + size_t(-1 - it.src1) * (P * C));
        __syncthreads();
        if (binary) kloop<MTW, NT, 8, XS, true>(acc, uaddr, ring1, w1row2, w1row2);
        __syncthreads();
        if (binary) {                                     // ReLU(acc) -> bf16 -> centre of the halo tile (in place)
#pragma unroll
            for (int t = 0; t < MTW; ++t)
                if (t * 32 + r < UPIX) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const u32x4 pk = packed(t, nt, q);
                            *reinterpret_cast<u32x4*>(lds_raw + uaddr[t] - uint32_t(h * 128) + CENTER +
                                                      uint32_t((chan(nt) + q * 8) * 2)) = pk;
                            // (half-node layouts: the two windows overlap; both write the same values there)
                            if constexpr (KEEP)
                                *reinterpret_cast<u32x4*>(a.keep_u + (size_t(a.first_item + first + node_local) * P + urow0 * S + t * 32 + r) * C +
                                                          chan(nt) + q * 8) = pk;
                        }
                }
        }
        __syncthreads();
    }

    // ---- first conv3x3 + ReLU, result replaces the tile; the old centre values become the residual
    PHASE(3);
    if (active) {
        if (!DEEP || a.any_binary) ring_fill<NT, RW>(ring, wrow_a);   // (after the 1x1 convolution, whose loops need the registers)
        init_bias(a.b3a);
        kloop<MTW, NT, RW, XS, false>(acc, xaddr, ring, wrow_a, wrow_b);   // leaves the ring filled for the second conv
    }
    PHASE(4);
    __syncthreads();
    PHASE(5);
    if (active) {
        auto bias8 = [&](int ch, f32x4& lo, f32x4& hi) {
            lo = f32x4{0.f, 0.f, 0.f, 0.f};
            hi = lo;
            if (a.b3b) {
                const float* bp = a.b3b + size_t(it.type) * C + ch;
                lo = *reinterpret_cast<const f32x4*>(bp);
                hi = *reinterpret_cast<const f32x4*>(bp + 4);
            }
        };
        // acc[t][nt][8q .. 8q+7]: ReLU'd bf16 into the tile, old centre values + bias back into acc
        auto swap8 = [&](int t, int nt, int q, const f32x4& blo, const f32x4& bhi) {
            const uint32_t addr = centre(t) + uint32_t((chan(nt) + q * 8) * 2);
            const u32x4 res = *reinterpret_cast<const u32x4*>(lds_raw + addr);
            const u32x4 pk = packed(t, nt, q);
            *reinterpret_cast<u32x4*>(lds_raw + addr) = pk;
            if constexpr (KEEP)
                *reinterpret_cast<u32x4*>(a.keep_m + (size_t(a.first_item + first + node_local) * P + wrow0 * S + t * 32 + r) * C +
                                          chan(nt) + q * 8) = pk;
            acc[t][nt][8 * q + 0] = __uint_as_float(res.x << 16) + blo.x;
            acc[t][nt][8 * q + 1] = __uint_as_float(res.x & 0xffff0000u) + blo.y;
            acc[t][nt][8 * q + 2] = __uint_as_float(res.y << 16) + blo.z;
            acc[t][nt][8 * q + 3] = __uint_as_float(res.y & 0xffff0000u) + blo.w;
            acc[t][nt][8 * q + 4] = __uint_as_float(res.z << 16) + bhi.x;
            acc[t][nt][8 * q + 5] = __uint_as_float(res.z & 0xffff0000u) + bhi.y;
            acc[t][nt][8 * q + 6] = __uint_as_float(res.w << 16) + bhi.z;
            acc[t][nt][8 * q + 7] = __uint_as_float(res.w & 0xffff0000u) + bhi.w;
        };
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                f32x4 blo, bhi;
                bias8(chan(nt) + q * 8, blo, bhi);
#pragma unroll
                for (int t = 0; t < MTW; ++t)
                    if (t * 32 + r < NPIX) swap8(t, nt, q, blo, bhi);
            }
    }
    PHASE(6);
    __syncthreads();
    PHASE(7);

    // ---- second conv3x3 on top of (residual + bias), ReLU, scatter
    if (active) {
        kloop<MTW, NT, RW, XS, false>(acc, xaddr, ring, wrow_b, wrow_b);
        PHASE(8);
        bf16_t* dst = it.dst >= 0 ? a.slots + size_t(it.dst) * (P * C) : a.out + size_t(-1 - it.dst) * (P * C);
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            const int pl = t * 32 + r;
            const int p = wrow0 * S + pl;
            if (pl < NPIX && p >= orow0 * S && p < orow1 * S) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        *reinterpret_cast<u32x4*>(dst + size_t(p) * C + chan(nt) + q * 8) = packed(t, nt, q);
            }
        }
    }
    PHASE(9);
}

template <int WMODE, bool KEEP = false>
__global__ __launch_bounds__(256, WMODE == 4 ? 2 : 1) void k_module_mfma(MfArgs a)
{
    // Workgroup -> position in the launch group.  Consecutive workgroup ids land on different
    // XCDs; give every XCD one contiguous run of items (items are sorted by function id) so that
    // a function's weights stay in as few L2s as possible.
    const int per_xcd = gridDim.x >> 3;
    module_body<WMODE, true, KEEP>(a, (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3));
}

// ---- one dependency-driven launch per batch ---------------------------------------------------------
// Resident workgroups claim units of work (tickets) in the plan's execution order from one device
// counter.  A unit's arguments are results of units with smaller tickets; those were claimed by
// workgroups that are already running and that in turn only wait for still smaller tickets, so the unit
// with the smallest unfinished ticket never waits and every wait ends.  The waits are bounded all the
// same: a workgroup that gives up raises the status word, and from then on every workgroup only drains
// the counter.  ready[slot] counts published halves of a result (a whole node adds 2).
struct PersistArgs {
    const int32_t* tickets;   // device [n_tickets]: 4 * item + part
    int32_t n_tickets;
    int32_t spin_limit;
    int32_t* ready;           // device [n_slots], zero before the launch
    int32_t* counter;         // device, zero before the launch
    int32_t* status;          // device, zero before the launch; 1 = a wait expired
};

__device__ __forceinline__ int32_t load_relaxed(const int32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256, 1) void k_module_persist(MfArgs a, PersistArgs q)
{
    __shared__ int32_t s_ticket, s_go;
    const dynb_item* items = a.items;
    for (;;) {
        if (threadIdx.x == 0) {
            const int32_t tk = __hip_atomic_fetch_add(q.counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int32_t go = 0;                                   // 0: stop, 1: compute, 2: skip (draining after an error)
            if (tk < q.n_tickets) {
                go = 1;
                const dynb_item it = items[q.tickets[tk] >> 2];
                const int nsrc = a.arity[it.type];
                for (int s = 0; s < nsrc && go == 1; ++s) {
                    const int32_t src = s == 0 ? it.src0 : it.src1;
                    if (src < 0) continue;                    // an example's feature map: always there
                    int32_t polls = 0;
                    while (load_relaxed(q.ready + src) < 2) {
                        if (polls >= q.spin_limit || load_relaxed(q.status) != 0) {
                            __hip_atomic_store(q.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            go = 2;
                            break;
                        }
                        ++polls;
                        __builtin_amdgcn_s_sleep(8);
                    }
                }
                if (go == 1 && load_relaxed(q.status) != 0) go = 2;
                // The arguments' maps were written by other CUs, possibly behind another L2: drop what this CU's
                // vector cache and this L2 may still hold of those addresses.  One wave does it for the
                // workgroup (its waves share both caches); the others load only after the barrier below.
                if (go == 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            s_ticket = tk;
            s_go = go;
        }
        __syncthreads();
        const int32_t tk = s_ticket, go = s_go;
        __syncthreads();                                      // both are read before thread 0 writes them again
        if (go == 0) return;
        if (go == 2) continue;
        const int32_t t = q.tickets[tk];
        MfArgs b = a;
        b.items = items + (t >> 2);
        b.count = 1;
        b.any_binary = (a.arity[b.items[0].type] == 2);
        const int part = t & 3;
        if (part == 0) module_body<2, false>(b, 0);          // both layouts in one kernel: the shallow weight ring fits
        else module_body<3, false>(b, part - 1);
        // Publish: every wave waits until its stores of the result have reached the L2 (all waves of a
        // workgroup sit behind the same one), then one thread writes that L2's dirty lines back to memory,
        // where every CU can see them, and raises the flag (the agent-scope release does both).
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();                                      // also frees the LDS tile for the next unit
        const int32_t dst = b.items[0].dst;
        if (threadIdx.x == 0 && dst >= 0)
            __hip_atomic_fetch_add(q.ready + dst, part == 0 ? 2 : 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void k_fill_i32(int32_t* p, size_t n, int32_t v)
{
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += size_t(gridDim.x) * blockDim.x) p[i] = v;
}

size_t elt_bytes(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

bool fast_shape(const dynb_shape* s) { return s->dtype == DYNB_BF16 && s->C == 128 && s->H == 14 && s->W == 14; }

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t packed_weight_bytes(int n_types) { return dynb_fast_packed_weight_bytes(n_types); }

}  // namespace

#ifdef DYNB_PHASE_CLOCKS
extern "C" int dynb_debug_phase_clocks(void* device_buf)
{
    long long* p = static_cast<long long*>(device_buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_phase_clk), &p, sizeof(p)) == hipSuccess ? DYNB_OK : DYNB_E_HIP;
}
#endif

// Device buffer layout of an uploaded plan: items | leaf-root example ids | arity table | tickets
static size_t plan_items_bytes(const dynb_plan* p) { return dynb_plan_items_bytes(p); }
static size_t plan_leaf_bytes(const dynb_plan* p) { return dynb_plan_leaf_bytes(p); }
static size_t plan_arity_bytes(const dynb_plan* p) { return dynb_plan_arity_bytes(p); }
static size_t plan_ticket_bytes(const dynb_plan* p) { return dynb_plan_ticket_bytes(p); }

extern "C" size_t dynbatch_plan_device_bytes(const dynb_plan* p)
{
    if (!p) return 0;
    return dynb_plan_keep_tables(p).end + 256;
}

// Workspace tail of the dependency-driven launch: ready[n_slots] | counter | status (after the slots and,
// without prepared weights, the packed weights)
static size_t persist_sync_bytes(const dynb_plan* p) { return dynb_fast_sync_bytes(p); }

// offset of that tail: behind the slots and the room for packed weights
static size_t persist_sync_offset(const dynb_plan* p)
{
    return dynb_fast_sync_offset(p);
}

static std::atomic<int32_t> g_spin_limit{1 << 22};

extern "C" int32_t dynb_set_spin_limit(int32_t polls) { return g_spin_limit.exchange(polls < 0 ? 0 : polls); }

extern "C" int dynbatch_plan_upload(dynb_plan* p, void* dev_buf, size_t bytes, void* stream)
{
    if (!p || !dev_buf) return fail(DYNB_E_INVAL, "dynbatch_plan_upload: NULL argument");
    if (bytes < dynbatch_plan_device_bytes(p)) return fail(DYNB_E_WORKSPACE, "dynbatch_plan_upload: buffer too small");
    if (reinterpret_cast<uintptr_t>(dev_buf) & 15) return fail(DYNB_E_INVAL, "dynbatch_plan_upload: buffer not 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // One copy: the parts are laid out in a host image of the device buffer (a separate copy per part costs a few
    // microseconds of stream time each, which shows in a step of less than a millisecond).  The image belongs to the
    // plan, so it lives as long as the copy may need it.
    const dynb_keep_tables t = dynb_plan_keep_tables(p);
    p->image.assign(t.end, 0);
    char* h = p->image.data();
    auto put = [&](size_t at, const void* src, size_t n) { if (n) memcpy(h + at, src, n); };
    put(0, p->items.data(), p->items.size() * sizeof(dynb_item));
    put(plan_items_bytes(p), p->leaf_roots.data(), p->leaf_roots.size() * sizeof(int32_t));
    put(plan_items_bytes(p) + plan_leaf_bytes(p), p->arity.data(), p->arity.size());
    put(plan_items_bytes(p) + plan_leaf_bytes(p) + plan_arity_bytes(p), p->tickets.data(), p->tickets.size() * sizeof(int32_t));
    if (p->keep) {                                            // what the backward pass works from
        put(t.gdst0, p->grad_dst0.data(), p->grad_dst0.size() * 4);
        put(t.gdst1, p->grad_dst1.data(), p->grad_dst1.size() * 4);
        put(t.leaf_first, p->leaf_first.data(), p->leaf_first.size() * 4);
        put(t.root_item, p->root_item.data(), p->root_item.size() * 4);
        put(t.fn_items, p->fn_items.data(), p->fn_items.size() * 4);
        put(t.units, p->wg_units.data(), p->wg_units.size() * sizeof(dynb_wg_unit));
        put(t.groups, p->wg_groups.data(), p->wg_groups.size() * sizeof(dynb_wg_group));
        put(t.order, p->wg_order.data(), p->wg_order.size() * 4);
    }
    if (t.end) HIP_TRY(hipMemcpyAsync(dev_buf, h, t.end, hipMemcpyHostToDevice, st), "dynbatch_plan_upload");
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
    size_t bytes = align256(n * map);
    if (fast_shape(s)) bytes += align256(packed_weight_bytes(p->n_types));    // weights in MFMA fragment order
    if (fast_shape(s)) bytes += persist_sync_bytes(p);                        // ready flags, ticket counter, status
    if (fast_shape(s)) bytes += dynb_fast_keep_bytes(p);                      // u and mid of every item for the backward pass
    return std::max<size_t>(bytes, 256);
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
    const bool timed = dynb::timing_on(), coarse = dynb::timing_coarse();
    if (timed) dynb::timing_mark(st, dynb::ST_SETUP, 0);
    int32_t evals = 0;
    for (const dynb_launch& l : p->launches) {
        evals += l.count;
        a.items = reinterpret_cast<const dynb_item*>(d) + l.start;
        a.count = l.count;
        const bool any_binary = l.any_binary != 0;
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
        if (timed && !coarse) dynb::timing_mark(st, int32_t(&l - p->launches.data()), l.count);
    }
    if (coarse) dynb::timing_mark(st, 0, evals);
    HIP_TRY(hipGetLastError(), "dynbatch_execute(generic kernels)");
    return DYNB_OK;
}

// w1 (2 halves), w3a, w3b (9 taps each) -> fragment order at pk: [w3a | w3b | w1]
static void launch_pack(const dynb_module_weights* w, int n_types, char* pk, hipStream_t st)
{
    const size_t tap_bytes = size_t(n_types) * 128 * 128 * 2;
    const unsigned g9 = unsigned(std::min<size_t>((size_t(n_types) * 4 * 9 * 512 + 255) / 256, 4096));
    hipLaunchKernelGGL(k_pack_weights, dim3(g9), dim3(256), 0, st, static_cast<const u32x4*>(w->w3a),
                       reinterpret_cast<u32x4*>(pk), n_types, 9);
    hipLaunchKernelGGL(k_pack_weights, dim3(g9), dim3(256), 0, st, static_cast<const u32x4*>(w->w3b),
                       reinterpret_cast<u32x4*>(pk + 9 * tap_bytes), n_types, 9);
    if (w->w1)
        hipLaunchKernelGGL(k_pack_weights, dim3(g9), dim3(256), 0, st, static_cast<const u32x4*>(w->w1),
                           reinterpret_cast<u32x4*>(pk + 18 * tap_bytes), n_types, 2);
}

static int run_mfma(const dynb_plan* p, const dynb_module_weights* w, const void* feats, void* out, char* ws,
                    hipStream_t st)
{
    static std::atomic<uint64_t> attr_set{0};                 // one bit per device
    static int cu_count[64] = {};
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
    if (!(attr_set.load() >> (dev & 63) & 1)) {
        int cus = 0;
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute");
        cu_count[dev & 63] = cus > 0 ? cus : 256;
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_persist),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_persist)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<2>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<3>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<3>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<4>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<4>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<2, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<2, keep>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<3, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<3, keep>)");
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_module_mfma<4, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, mf::TILE_BYTES),
                "hipFuncSetAttribute(k_module_mfma<4, keep>)");
        attr_set.fetch_or(uint64_t(1) << (dev & 63));
    }
    const char* d = static_cast<const char*>(p->dev_buf);
    MfArgs a;
    a.arity = reinterpret_cast<const uint8_t*>(d + plan_items_bytes(p) + plan_leaf_bytes(p));
    a.feats = static_cast<const bf16_t*>(feats);
    a.out = static_cast<bf16_t*>(out);
    a.slots = reinterpret_cast<bf16_t*>(ws);
    // weights in fragment order: the caller's prepared copy, or a fresh one behind the slots
    // (about 0.6 MB per function)
    const size_t tap_bytes = size_t(p->n_types) * 128 * 128 * 2;
    char* pk = w->packed ? static_cast<char*>(const_cast<void*>(w->packed))
                         : ws + align256(size_t(p->n_slots) * mf::P * mf::C * 2);
    bf16_t* pk3a = reinterpret_cast<bf16_t*>(pk);
    bf16_t* pk3b = reinterpret_cast<bf16_t*>(pk + 9 * tap_bytes);
    bf16_t* pk1 = reinterpret_cast<bf16_t*>(pk + 18 * tap_bytes);
    if (!w->packed) launch_pack(w, p->n_types, pk, st);
    a.w1 = pk1; a.b1 = w->b1;
    a.w3a = pk3a; a.b3a = w->b3a;
    a.w3b = pk3b; a.b3b = w->b3b;
    a.first_item = 0;
    a.keep_u = a.keep_m = nullptr;
    if (p->keep) {
        a.keep_m = reinterpret_cast<bf16_t*>(ws + dynb_fast_keep_offset(p));
        a.keep_u = a.keep_m + p->items.size() * size_t(mf::P) * mf::C;
    }
    const bool timed = dynb::timing_on(), coarse = dynb::timing_coarse();
    if (p->persistent) {
        // one launch for the whole batch: clear the ready flags, the ticket counter and the status word with a
        // fill kernel (no memset node: the call may be captured into a graph), then the resident workgroups
        PersistArgs q;
        q.tickets = reinterpret_cast<const int32_t*>(d + plan_items_bytes(p) + plan_leaf_bytes(p) + plan_arity_bytes(p));
        q.n_tickets = int32_t(p->tickets.size());
        q.spin_limit = g_spin_limit.load();
        q.ready = reinterpret_cast<int32_t*>(ws + persist_sync_offset(p));
        q.counter = q.ready + p->n_slots;
        q.status = q.counter + 1;
        const size_t nsync = size_t(p->n_slots) + 2;
        hipLaunchKernelGGL(k_fill_i32, dim3(unsigned(std::min<size_t>((nsync + 255) / 256, 256))), dim3(256), 0, st, q.ready, nsync, 0);
        if (timed) dynb::timing_mark(st, dynb::ST_SETUP, 0);
        // a plan that also keeps u and mid for the backward pass runs one launch per label (below); its status
        // word stays clear
        if (!p->keep) {
            a.items = reinterpret_cast<const dynb_item*>(d);
            a.count = int32_t(p->items.size());
            a.any_binary = 0;
            const int resident = cu_count[dev & 63];          // one workgroup per CU (73 KB of LDS, all registers)
            const unsigned grid = unsigned(std::min<int>(q.n_tickets, resident));
            hipLaunchKernelGGL(k_module_persist, dim3(grid), dim3(256), mf::TILE_BYTES, st, a, q);
            if (timed) dynb::timing_mark(st, 0, a.count);
            HIP_TRY(hipGetLastError(), "dynbatch_execute(dependency-driven kernel)");
            return DYNB_OK;
        }
    }
    if (timed && !p->persistent) dynb::timing_mark(st, dynb::ST_SETUP, 0);
    int32_t evals = 0;
    for (const dynb_launch& l : p->launches) {
        evals += l.count;
        a.items = reinterpret_cast<const dynb_item*>(d) + l.start;
        a.first_item = l.start;
        a.count = l.count;
        a.any_binary = l.any_binary;
        // half a node per workgroup while that still fits the chip's 256 CUs in one round, one node per
        // workgroup up to 256 nodes; beyond that, and whenever several batches are in flight (their narrow
        // groups share the chip), the 256-register variant with two workgroups per CU
        int wm = (p->throughput || l.count > 256) ? 4 : (l.count <= 128) ? 3 : 2;
#ifdef DYNB_PHASE_CLOCKS
        if (const char* f = getenv("DYNB_FORCE_WM")) wm = atoi(f);
#endif
        const int nwg = (wm == 3) ? 2 * l.count : l.count;
        const unsigned grid = unsigned((nwg + 7) / 8 * 8);
        if (p->keep) {
            if (wm == 4)
                hipLaunchKernelGGL((k_module_mfma<4, true>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
            else if (wm == 3)
                hipLaunchKernelGGL((k_module_mfma<3, true>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
            else
                hipLaunchKernelGGL((k_module_mfma<2, true>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
        } else if (wm == 4)
            hipLaunchKernelGGL((k_module_mfma<4>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
        else if (wm == 3)
            hipLaunchKernelGGL((k_module_mfma<3>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
        else
            hipLaunchKernelGGL((k_module_mfma<2>), dim3(grid), dim3(256), mf::TILE_BYTES, st, a);
        if (timed && !coarse) dynb::timing_mark(st, int32_t(&l - p->launches.data()), l.count);
    }
    if (coarse) dynb::timing_mark(st, 0, evals);
    HIP_TRY(hipGetLastError(), "dynbatch_execute(mfma kernels)");
    return DYNB_OK;
}

extern "C" size_t dynbatch_packed_weights_bytes(const dynb_shape* s, int32_t n_types)
{
    if (!s || n_types <= 0 || !fast_shape(s)) return 0;
    return align256(packed_weight_bytes(n_types));
}

extern "C" int dynbatch_pack_weights(const dynb_shape* s, int32_t n_types, const dynb_module_weights* w, void* packed,
                                     size_t packed_bytes, void* stream)
{
    if (!s || !w || !packed || n_types <= 0) return fail(DYNB_E_INVAL, "dynbatch_pack_weights: NULL argument or n_types <= 0");
    if (!fast_shape(s)) return fail(DYNB_E_UNSUPPORTED, "dynbatch_pack_weights: this shape has no packed layout");
    if (!w->w3a || !w->w3b) return fail(DYNB_E_INVAL, "dynbatch_pack_weights: conv3x3 weights missing");
    if (reinterpret_cast<uintptr_t>(packed) & 255) return fail(DYNB_E_INVAL, "dynbatch_pack_weights: buffer not 256-byte aligned");
    if (packed_bytes < dynbatch_packed_weights_bytes(s, n_types))
        return fail(DYNB_E_WORKSPACE, "dynbatch_pack_weights: buffer too small");
    launch_pack(w, n_types, static_cast<char*>(packed), static_cast<hipStream_t>(stream));
    HIP_TRY(hipGetLastError(), "dynbatch_pack_weights");
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

extern "C" int dynbatch_execute_check(const dynb_plan* p, const dynb_shape* s, const void* workspace, void* stream)
{
    if (!p || !s || !workspace) return fail(DYNB_E_INVAL, "dynbatch_execute_check: NULL argument");
    if (!p->persistent) return fail(DYNB_E_INVAL, "dynbatch_execute_check: the plan was not made with DYNB_PLAN_PERSISTENT");
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(hipStreamSynchronize(st), "dynbatch_execute_check(synchronize)");
    if (!fast_shape(s) || p->items.empty()) return DYNB_OK;   // those run one launch per label: nothing waits
    int32_t status = 0;
    const char* w = static_cast<const char*>(workspace) + persist_sync_offset(p) + (size_t(p->n_slots) + 1) * sizeof(int32_t);
    HIP_TRY(hipMemcpy(&status, w, sizeof(status), hipMemcpyDeviceToHost), "dynbatch_execute_check(read status)");
    if (status != 0)
        return fail(DYNB_E_HIP, "dynbatch_execute: a workgroup gave up waiting for an argument of its node; the results are invalid");
    return DYNB_OK;
}
