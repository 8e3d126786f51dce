// Sparsely gated mixture-of-experts layer with the paper's degenerate one-level batching
// (Results / Sparsely Gated Mixture of Experts): the k*b expert uses known after gating are
// grouped by expert so that each of the n experts is called once on its stacked rows.
//
// Stages (all on the caller's stream, no host synchronisation):
//   gate      logits = x Wg^T + noise * softplus(x Wn^T)                 MFMA, fp32 accumulate
//   top-k     k largest per token (ties -> lower expert), softmax        one wave per token
//   group     stable counting sort of the T*k uses by expert             rank-by-prefix-sum, no
//                                                                        order-dependent atomics
//   permute   xs[inv[t*k+j]] = x[t]  (= xs[pos] = x[perm[pos] / k])       HBM-bound scatter
//   experts   hid = ReLU(xs W1_e^T), y = hid W2_e^T per group             grouped MFMA GEMM, ragged
//                                                                        and empty groups allowed
//   combine   out[t] = sum_j w[t][j] * y[inv[t*k+j]]                      HBM-bound, fixed order
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <type_traits>
#include <mutex>
#include <string>
#include <vector>

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

constexpr int SORT_BLOCK = 256;   // uses ranked together by one workgroup
constexpr int TM = 64;            // rows of one grouped-GEMM tile
constexpr int TN = 256;           // output features of one grouped-GEMM tile
constexpr int NTW = TN / 64;      // 16-feature sub-tiles per wave (4 waves split the features)
constexpr int MAX_K = 8;          // uses of a token whose places are kept in registers (more are looked up)
constexpr int MG = 8;             // row tiles of one expert that walk the feature tiles together
constexpr int XCD_CHUNK = 128;    // consecutive grouped-GEMM tiles dealt to one XCD

__device__ __forceinline__ bf16x8 ldg_frag(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

// ------------------------------------------------------------------------------------------ gate
// Workgroup tile: 64 tokens x 64 experts, both gate matrices at once.  Operands are staged through
// LDS in K-chunks of 64 with coalesced 128-byte row reads (see the grouped GEMM below for why), the
// next chunk is prefetched into registers.  A wave owns a 32-token x 32-expert quarter of the tile
// for both matrices (clean and noise accumulators), multiplied with 32x32x16 MFMAs.
constexpr int GKC = 64;                // K-chunk
constexpr int GLDP = GKC + 8;          // LDS row pitch in elements (144 bytes, conflict free)

// softplus(z) = max(z, 0) + log(1 + u), u = exp(-|z|) in (0, 1], from the hardware's exp2 and log2 (good to about
// 1e-7).  w = 1 + u is rounded; c = u - (w - 1) is exactly what the rounding dropped (w - 1 and the difference are
// exact for w in [1, 2]), and log(1 + u) = log(w) + c / w, where leaving out the division costs less than 2^-25: small
// u keep their relative accuracy without a second code path (u < 2^-24 gives w = 1, log(w) = 0, c = u).
__device__ __forceinline__ float softplus_f(float z)
{
    const float u = __builtin_amdgcn_exp2f(-1.4426950408889634f * fabsf(z));
    const float w = 1.f + u;
    const float c = u - (w - 1.f);
    return fmaxf(z, 0.f) + fmaf(0.6931471805599453f, __builtin_amdgcn_logf(w), c);
}

__global__ __launch_bounds__(256) void k_gate(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wg,
                                              const bf16_t* __restrict__ Wn, const float* __restrict__ noise,
                                              float* __restrict__ logits, int T, int d, int E)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ws[128 * GLDP];   // rows 0..63 Wg, 64..127 Wn
    __shared__ __attribute__((aligned(16))) bf16_t Xs[64 * GLDP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int t0 = blockIdx.y * 64, e0 = blockIdx.x * 64;
    const int part = tid & 7, srow = tid >> 3;          // staging: 32 rows x 8 pieces of 16 bytes per pass
    const bf16_t* wsrc[4];
    const bf16_t* xsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const size_t row = size_t(min(e0 + srow + i * 32, E - 1)) * d + part * 8;
        wsrc[i] = Wg + row;
        wsrc[2 + i] = (noise ? Wn : Wg) + row;
        xsrc[i] = x + size_t(min(t0 + srow + i * 32, T - 1)) * d + part * 8;
    }
    u32x4 wreg[4], xreg[2];
    auto fetch = [&](int kc) {
        const bool inside = kc * GKC + part * 8 < d;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            wreg[i] = inside ? *reinterpret_cast<const u32x4*>(wsrc[i] + kc * GKC) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 2; ++i)
            xreg[i] = inside ? *reinterpret_cast<const u32x4*>(xsrc[i] + kc * GKC) : u32x4{0u, 0u, 0u, 0u};
    };
    // 4 waves = 2 token halves x 2 expert halves; each wave one 32 x 32 tile per gate matrix (32x32x16 MFMAs)
    const int q = lane & 31, hk = lane >> 5, th = wave & 1, eh = wave >> 1;
    f32x16 ag, an;
#pragma unroll
    for (int i = 0; i < 16; ++i) { ag[i] = 0.f; an[i] = 0.f; }
    const int nchunk = (d + GKC - 1) / GKC;
    fetch(0);
    for (int kc = 0; kc < nchunk; ++kc) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(Ws + (srow + i * 32) * GLDP + part * 8) = wreg[i];
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4*>(Xs + (srow + i * 32) * GLDP + part * 8) = xreg[i];
        __syncthreads();
        if (kc + 1 < nchunk) fetch(kc + 1);
#pragma unroll
        for (int ks = 0; ks < GKC / 16; ++ks) {
            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(Xs + (th * 32 + q) * GLDP + ks * 16 + hk * 8);
            const bf16x8 gf = *reinterpret_cast<const bf16x8*>(Ws + (eh * 32 + q) * GLDP + ks * 16 + hk * 8);
            ag = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, gf, ag, 0, 0, 0);
            if (noise) {
                const bf16x8 nf = *reinterpret_cast<const bf16x8*>(Ws + (64 + eh * 32 + q) * GLDP + ks * 16 + hk * 8);
                an = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, nf, an, 0, 0, 0);
            }
        }
        __syncthreads();
    }
    // lane holds expert e0 + eh*32 + q, tokens t0 + th*32 + 8*(i/4) + 4*hk + i%4 in element i
    const int e = e0 + eh * 32 + q;
    if (e >= E) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int t = t0 + th * 32 + 8 * (i / 4) + 4 * hk + (i % 4);
        if (t >= T) continue;
        float v = ag[i];
        if (noise) {
            const float z = an[i];
            const float sp = softplus_f(z);
            v += noise[size_t(t) * E + e] * sp;
        }
        logits[size_t(t) * E + e] = v;
    }
}

// The same product for wide gates: a workgroup owns a CU and a tile of 256 tokens x 128 experts, both gate matrices
// at once.  A 64 x 64 tile takes in 24 KB per K-chunk for 8 MFMAs per wave (96 B per MFMA clock), three times what
// a CU receives from L2; this tile takes in 64 KB for 64 MFMAs per wave (32 B per MFMA clock).  Operands go through LDS in K-chunks of 64, double buffered, one barrier per chunk.  A wave owns 128
// tokens x 64 experts of both matrices: 16 accumulator tiles.  It is alone on its SIMD, so nothing but its own
// instruction order hides latency: every request is issued between two MFMA groups - an LDS fragment of the next
// K-step; a 16-byte piece of chunk c+1 going from its register to the other LDS buffer, and the piece of chunk c+2
// that takes its place; during the last four chunks half of the epilogue's noise values.  Tiles that share token
// rows are given to one die: its L2 keeps the rows, and the gate matrices too.  Whole tiles only: E a multiple of
// 128, d of 64 and at least 256; the tokens behind the last whole tile of 256, and every other shape, go to k_gate.
constexpr int GB_TOK = 256, GB_EXP = 128;
constexpr int GB_BUF = (GB_TOK + 2 * GB_EXP) * GLDP;       // elements of one LDS buffer: x rows, Wg rows, Wn rows
constexpr int GB_LDS_BYTES = 2 * GB_BUF * 2;

template <bool NOISY>
__global__ __launch_bounds__(256, 1) void k_gate_big(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wg,
                                                     const bf16_t* __restrict__ Wn, const float* __restrict__ noise,
                                                     float* __restrict__ logits, int T, int d, int E, int n_tok_tiles, int n_exp_tiles,
                                                     int tok_tiles_per_die)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char gb_lds[];
    const int die = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int tok_tile = die * tok_tiles_per_die + j / n_exp_tiles, exp_tile = j % n_exp_tiles;
    if (j / n_exp_tiles >= tok_tiles_per_die || tok_tile >= n_tok_tiles) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int t0 = tok_tile * GB_TOK, e0 = exp_tile * GB_EXP;
    const int part = tid & 7, srow = tid >> 3;          // staging: 32 rows x 8 pieces of 16 bytes per pass
    constexpr int NP = NOISY ? 16 : 12;                 // pieces of a chunk per thread: 8 of x, 4 of Wg, 4 of Wn
    constexpr int NF = NOISY ? 8 : 6;                   // fragments of a K-step: 4 token tiles, 2 (+2) expert tiles
    const int q = lane & 31, hk = lane >> 5, th = wave & 1, eh = wave >> 1;   // 2 token halves x 2 expert halves
    bf16_t* const lds = reinterpret_cast<bf16_t*>(gb_lds);

    // piece i of a chunk: 16 bytes of row srow + 32 i of the x tile (i < 8), of the Wg tile (i < 12), of the Wn tile;
    // 32-bit offsets from the tiles' corners, one register for all of them (a tile spans 256 d < 2^31 elements)
    const bf16_t* const x_tile = x + size_t(t0) * d;
    const bf16_t* const wg_tile = Wg + size_t(e0) * d;
    const bf16_t* const wn_tile = NOISY ? Wn + size_t(e0) * d : nullptr;
    // (byte offsets: a uniform base plus a 32-bit lane offset is an addressing mode of the loads and stores)
    const unsigned row_bytes = unsigned(d) * 2u, lane_off = unsigned(srow) * row_bytes + unsigned(part * 16);
    u32x4 stage[NP];                                    // a chunk on its way to LDS
    auto fetch_piece = [&](int i, int kc) {
        const char* src = reinterpret_cast<const char*>(i < 8 ? x_tile : i < 12 ? wg_tile : wn_tile);
        const unsigned row32 = unsigned(i < 8 ? i : (i - 8) & 3) * 32u;
        stage[i] = *reinterpret_cast<const u32x4*>(src + (lane_off + row32 * row_bytes + unsigned(kc * GKC * 2)));
    };
    auto store_piece = [&](int i, bf16_t* buf) {        // piece i covers rows srow + 32 i of the buffer's 512
        *reinterpret_cast<u32x4*>(buf + (srow + i * 32) * GLDP + part * 8) = stage[i];
    };
    // element i of accumulator tile n = 4 b + a (expert column b, token tile a) belongs to expert e0 + eh*64 + b*32
    // + q and token t0 + th*128 + a*32 + 4*hk + 8*(i/4) + i%4; its place in the tile of logits (and of noise values)
    // is a 32-bit byte offset from the tile's corner
    const unsigned uE = unsigned(E) * 4u;                 // bytes of a row of logits
    const unsigned lane_at = unsigned(th * 128 + 4 * hk) * uE + unsigned(eh * 64 + q) * 4u;
    auto at = [&](int n, int i) { return lane_at + unsigned((n & 3) * 32 + 8 * (i / 4) + (i % 4)) * uE + unsigned((n >> 2) * 128); };
    const char* const noise_tile = NOISY ? reinterpret_cast<const char*>(noise + size_t(t0) * E + e0) : nullptr;
    float nz[NOISY ? 8 : 1][16];                          // noise values, 16 per accumulator tile

    f32x16 ag[4][2], an[NOISY ? 4 : 1][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) { ag[a][b][i] = 0.f; if (NOISY) an[NOISY ? a : 0][b][i] = 0.f; }

    // one chunk: 4 K-steps of 8 MFMA groups (a token tile x an expert tile, both matrices); `side(g)` issues what
    // else has to be requested before group g, g = 0..31
    auto chunk = [&](const bf16_t* buf, auto&& side) {
        const bf16_t* Xs = buf;
        const bf16_t* Ws = buf + GB_TOK * GLDP;          // rows 0..127 Wg, 128..255 Wn
        auto read_frag = [&](int r, int ks) -> bf16x8 {
            const bf16_t* row = r < 4   ? Xs + (th * 128 + r * 32 + q) * GLDP
                                : r < 6 ? Ws + (eh * 64 + (r - 4) * 32 + q) * GLDP
                                        : Ws + (GB_EXP + eh * 64 + (r - 6) * 32 + q) * GLDP;
            return *reinterpret_cast<const bf16x8*>(row + ks * 16 + hk * 8);
        };
        bf16x8 fr[2][NF];
#pragma unroll
        for (int r = 0; r < NF; ++r) fr[0][r] = read_frag(r, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < GKC / 16; ++ks) {
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const int a = g >> 1, b = g & 1;
                if (ks + 1 < GKC / 16 && g < NF) fr[(ks + 1) & 1][g] = read_frag(g, ks + 1);
                side(ks * 8 + g);
                __builtin_amdgcn_sched_barrier(0);
                ag[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ks & 1][a], fr[ks & 1][4 + b], ag[a][b], 0, 0, 0);
                if (NOISY)
                    an[NOISY ? a : 0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ks & 1][a], fr[ks & 1][NOISY ? 6 + b : 0],
                                                                                  an[NOISY ? a : 0][b], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    const int nchunk = d / GKC;
#pragma unroll
    for (int i = 0; i < NP; ++i) fetch_piece(i, 0);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        store_piece(i, lds);
        fetch_piece(i, min(1, nchunk - 1));
    }
    __syncthreads();
    // chunk kc multiplies out of buffer kc & 1 while chunk kc+1 moves from the registers to the other buffer (all
    // waves left that buffer before the last barrier) and chunk kc+2 is requested into the registers; past the end
    // the requests repeat the last chunk, which nobody reads.  The last four chunks also request the noise values
    // of accumulator tiles 0..3, one tile each: every workgroup of the launch reaches its epilogue at about the
    // same time, and what they all ask of HBM then is what bounds the epilogue.
    auto steady = [&](int kc, auto&& also) {
        bf16_t* other = lds + ((kc + 1) & 1) * GB_BUF;
        const int k2 = min(kc + 2, nchunk - 1);
        chunk(lds + (kc & 1) * GB_BUF, [&](int g) {
            if ((g >> 1) < NP) {
                if ((g & 1) == 0) store_piece(g >> 1, other);
                else fetch_piece(g >> 1, k2);
            }
            also(g);
        });
        __syncthreads();
    };
    auto noise_of = [&](auto n) {                     // tile n's 16 values, in the even groups
        return [&, n](int g) {
            if (NOISY && (g & 1) == 0) nz[NOISY ? decltype(n)::value : 0][g >> 1] = *reinterpret_cast<const float*>(noise_tile + at(decltype(n)::value, g >> 1));
        };
    };
    for (int kc = 0; kc + 4 < nchunk; ++kc) steady(kc, [](int) {});
    steady(nchunk - 4, noise_of(std::integral_constant<int, 0>{}));
    steady(nchunk - 3, noise_of(std::integral_constant<int, 1>{}));
    steady(nchunk - 2, noise_of(std::integral_constant<int, 2>{}));
    chunk(lds + ((nchunk - 1) & 1) * GB_BUF, noise_of(std::integral_constant<int, 3>{}));

    // the noise values of tile n+4 are requested before tile n is worked on
    char* const tile = reinterpret_cast<char*>(logits + size_t(t0) * E + e0);
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        const int a = n & 3, b = n >> 2;
        if (NOISY && n + 4 < 8) {
#pragma unroll
            for (int i = 0; i < 16; ++i) nz[NOISY ? n + 4 : 0][i] = *reinterpret_cast<const float*>(noise_tile + at(n + 4, i));
            __builtin_amdgcn_sched_barrier(0);
        }
        // a wave alone on its SIMD waits out every dependent instruction, so the softplus of 8 elements advances
        // stage by stage
#pragma unroll
        for (int i0 = 0; i0 < 16; i0 += 8) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = ag[a][b][i0 + i];
            if (NOISY) {
                float z[8], u[8], w[8], c[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) z[i] = an[NOISY ? a : 0][b][i0 + i];
#pragma unroll
                for (int i = 0; i < 8; ++i) u[i] = __builtin_amdgcn_exp2f(-1.4426950408889634f * fabsf(z[i]));
#pragma unroll
                for (int i = 0; i < 8; ++i) w[i] = 1.f + u[i];
#pragma unroll
                for (int i = 0; i < 8; ++i) c[i] = u[i] - (w[i] - 1.f);
#pragma unroll
                for (int i = 0; i < 8; ++i) w[i] = __builtin_amdgcn_logf(w[i]);
#pragma unroll
                for (int i = 0; i < 8; ++i) c[i] = __builtin_amdgcn_fmed3f(z[i], 0.f, INFINITY) + fmaf(0.6931471805599453f, w[i], c[i]);
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = fmaf(nz[NOISY ? n : 0][i0 + i], c[i], v[i]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) *reinterpret_cast<float*>(tile + at(n, i0 + i)) = v[i];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ------------------------------------------------------------------------------------------ top-k
// One wave per token. Selection compares fp32 logits exactly: larger first, equal -> lower id.
// The row is read once into registers (lane l holds experts l, l+64, ...; up to NV*64 experts) and the
// k selection rounds run on registers with a wave-wide argmax; NV = 0 re-reads the row every round
// (any E).  Selections come out in strictly descending (value, then ascending id) order, so "already
// taken" is simply "not below the previous selection": no list of chosen ids is kept and k may be
// anything up to E.  A NaN logit counts as -inf.
template <int NV>
__global__ __launch_bounds__(256) void k_topk(const float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                              float* __restrict__ topk_w, int T, int E, int k)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float* row = logits + size_t(t) * E;
    auto clean = [](float v) -> float { return v != v ? -INFINITY : v; };
    float reg[NV > 0 ? NV : 1];
    if (NV > 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int e = lane + 64 * i;
            reg[i] = e < E ? clean(row[e]) : 0.f;
        }
    }
    constexpr int NONE = 0x7fffffff;
    float last_v = INFINITY, v0 = 0.f, den = 0.f;
    int last_e = -1;
    int32_t* idx_t = topk_idx + size_t(t) * k;
    float* w_t = topk_w + size_t(t) * k;
    for (int j = 0; j < k; ++j) {
        float bv = -INFINITY;
        int bi = NONE;
        auto offer = [&](float v, int e) {
            const bool open = v < last_v || (v == last_v && e > last_e);       // below the previous selection
            if (open && (v > bv || bi == NONE)) { bv = v; bi = e; }
        };
        if (NV > 0) {
#pragma unroll
            for (int i = 0; i < NV; ++i)
                if (lane + 64 * i < E) offer(reg[i], lane + 64 * i);
        } else {
            for (int e = lane; e < E; e += 64) offer(clean(row[e]), e);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oi = __shfl_xor(bi, off);
            if (oi != NONE && (bi == NONE || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
        }
        // k <= E: a candidate always exists.  The selection is uniform over the wave.
        last_v = bv;
        last_e = bi;
        if (j == 0) v0 = bv;
        den += expf(bv - v0);
        if ((j & 63) == lane) { idx_t[j] = bi; w_t[j] = bv; }                  // raw logit until den is complete
    }
    for (int j = lane; j < k; j += 64) w_t[j] = expf(w_t[j] - v0) / den;       // each lane revisits its own stores
}

// The same selection for k <= MAX_K with the row in registers, as integer keys whose order is the logits' order
// (-0 is read as +0, NaN as -infinity, like above).  A round finds the largest key of the wave (per lane, then
// across lanes with data-parallel-primitive moves: inside rows of 16, then two row broadcasts to lane 63), and then
// its owner: the registers are asked in turn which lanes hold that key; the registers go up through the expert ids
// in groups of 256, so the first group with an answer holds the lowest expert id, the tie rule.  The owner replaces
// the key by one below every key a logit can have.  All of this is the same for the whole wave, so the search is
// scalar branches around one compare per register.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int wave_max_step(int v)
{
    // lanes without a source see the smallest integer, the identity of the maximum (which lets the move fold into it)
    return max(v, __builtin_amdgcn_update_dpp(int(0x80000000), v, CTRL, ROW_MASK, 0xF, false));
}

template <int NV>
__global__ __launch_bounds__(256) void k_topk_small(const float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w, int T, int E, int k)
{
    static_assert(NV % 4 == 0, "registers in groups of four consecutive experts");
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float* row = logits + size_t(t) * E;
    constexpr int TAKEN = int(0x80000000);           // below the key of -infinity (0x807fffff)
    // register 4 i + c holds expert 256 i + 4 lane + c: one 16-byte load per i where the row allows it
    int key[NV];
    const bool wide = (E & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;   // rows start 16-byte aligned, end on a group
    const bool full = E == 64 * NV;                   // no register lies beyond the row
#pragma unroll
    for (int i = 0; i < NV / 4; ++i) {
        const int e0 = 256 * i + 4 * lane;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (wide) {
            if (full || e0 < E) { const f32x4 q = *reinterpret_cast<const f32x4*>(row + e0); v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3]; }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) if (e0 + c < E) v[c] = row[e0 + c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float u = fmaxf(v[c], -INFINITY) + 0.f;            // the maximum drops a NaN, the sum turns -0 into +0
            const int bits = __builtin_bit_cast(int, u);
            const int ordered = bits ^ ((bits >> 31) & 0x7fffffff);
            key[4 * i + c] = (full || e0 + c < E) ? ordered : TAKEN;
        }
    }
    int chosen[MAX_K];
    float val[MAX_K];
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) { chosen[j] = -1; val[j] = 0.f; }
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
        if (j < k) {
            int m = key[0];
#pragma unroll
            for (int i = 1; i < NV; ++i) m = max(m, key[i]);
            m = wave_max_step<0xB1, 0xF>(m);       // quad_perm [1,0,3,2]
            m = wave_max_step<0x4E, 0xF>(m);       // quad_perm [2,3,0,1]
            m = wave_max_step<0x141, 0xF>(m);      // row_half_mirror
            m = wave_max_step<0x140, 0xF>(m);      // row_mirror
            m = wave_max_step<0x142, 0xA>(m);      // row_bcast15 into rows 1 and 3
            m = wave_max_step<0x143, 0xC>(m);      // row_bcast31 into rows 2 and 3
            m = __builtin_amdgcn_readlane(m, 63);
            bool found = false;
#pragma unroll
            for (int i = 0; i < NV / 4; ++i) {
                if (!found) {
                    int best = 0x7fffffff;           // lowest expert id of this group of 256 that holds m
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const unsigned long long owners = __ballot(key[4 * i + c] == m);
                        if (owners) best = min(best, 256 * i + 4 * (__ffsll(owners) - 1) + c);
                    }
                    if (best != 0x7fffffff) {
                        chosen[j] = best;
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (256 * i + 4 * lane + c == best) key[4 * i + c] = TAKEN;
                        found = true;
                    }
                }
            }
            const int bits = m ^ ((m >> 31) & 0x7fffffff);
            val[j] = __builtin_bit_cast(float, bits);
        }
    }
    // softmax over the k kept logits with the hardware's exp2 (arguments <= 0, results in (0, 1], good to ~2e-6)
    float den = 0.f, ex[MAX_K];
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
        ex[j] = j < k ? __expf(val[j] - val[0]) : 0.f;
        den += ex[j];
    }
#pragma unroll
    for (int j = 0; j < MAX_K; ++j)
        if (j < k && lane == j) {
            topk_idx[size_t(t) * k + j] = chosen[j];
            topk_w[size_t(t) * k + j] = ex[j] / den;
        }
}

// ------------------------------------------------------------------------------------------ grouping
__global__ void k_zero_i32(int32_t* p, size_t n)
{
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += size_t(gridDim.x) * blockDim.x) p[i] = 0;
}

// Block b ranks its 256 uses: lrank[a] = number of earlier uses in the block with the same expert;
// blockcnt[e][b] = uses of expert e in block b (written by the last such use; array pre-zeroed).
__global__ __launch_bounds__(SORT_BLOCK) void k_rank_blocks(const int32_t* __restrict__ idx, int32_t* __restrict__ lrank,
                                                            int32_t* __restrict__ blockcnt, int A, int nblk)
{
    __shared__ int32_t se[SORT_BLOCK];
    const int a = blockIdx.x * SORT_BLOCK + threadIdx.x;
    const int e = a < A ? idx[a] : -1;
    se[threadIdx.x] = e;
    __syncthreads();
    if (a >= A) return;
    int before = 0, total = 0;
    for (int j = 0; j < SORT_BLOCK; ++j) {
        const bool same = (se[j] == e);
        total += same;
        before += same && (j < int(threadIdx.x));
    }
    lrank[a] = before;
    if (before == total - 1) blockcnt[size_t(e) * nblk + blockIdx.x] = total;
}

// One wave per expert: exclusive scan of blockcnt[e][:] in place, counts[e] = total.
__global__ __launch_bounds__(256) void k_scan_blocks(int32_t* __restrict__ blockcnt, int32_t* __restrict__ counts,
                                                     int E, int nblk)
{
    const int lane = threadIdx.x & 63;
    const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= E) return;
    int32_t* col = blockcnt + size_t(e) * nblk;
    int carry = 0;
    for (int b0 = 0; b0 < nblk; b0 += 64) {
        const int b = b0 + lane;
        const int v = b < nblk ? col[b] : 0;
        int inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (b < nblk) col[b] = carry + inc - v;
        carry += __shfl(inc, 63);
    }
    if (lane == 0) counts[e] = carry;
}

// One workgroup of 16 waves: offsets = exclusive scan of counts; tile_start = exclusive scan of ceil(counts / TM).
// 1024 experts per pass: a scan inside every wave, the waves' totals through LDS.
constexpr int OFFS_THREADS = 1024;
__global__ __launch_bounds__(OFFS_THREADS) void k_offsets(const int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                          int32_t* __restrict__ tile_start, int E)
{
    __shared__ int32_t wsum[OFFS_THREADS / 64], wtsum[OFFS_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int carry = 0, tcarry = 0;
    for (int e0 = 0; e0 < E; e0 += OFFS_THREADS) {
        const int e = e0 + tid;
        const int c = e < E ? counts[e] : 0;
        const int tl = (c + TM - 1) / TM;
        int inc = c, tinc = tl;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(inc, off);
            const int to = __shfl_up(tinc, off);
            if (lane >= off) { inc += o; tinc += to; }
        }
        if (lane == 63) { wsum[wave] = inc; wtsum[wave] = tinc; }
        __syncthreads();
        int before = 0, tbefore = 0, all = 0, tall = 0;      // totals of the waves before this one, and of all
#pragma unroll
        for (int w = 0; w < OFFS_THREADS / 64; ++w) {
            const int a = wsum[w], t = wtsum[w];
            if (w < wave) { before += a; tbefore += t; }
            all += a;
            tall += t;
        }
        if (e < E) { offsets[e] = carry + before + inc - c; tile_start[e] = tcarry + tbefore + tinc - tl; }
        carry += all;
        tcarry += tall;
        __syncthreads();                                     // the totals are overwritten by the next pass
    }
    if (tid == 0) { offsets[E] = carry; tile_start[E] = tcarry; }
}

__global__ __launch_bounds__(SORT_BLOCK) void k_place(const int32_t* __restrict__ idx, const int32_t* __restrict__ lrank,
                                                      const int32_t* __restrict__ blockoff, const int32_t* __restrict__ offsets,
                                                      int32_t* __restrict__ perm, int32_t* __restrict__ inv, int A, int nblk)
{
    const int a = blockIdx.x * SORT_BLOCK + threadIdx.x;
    if (a >= A) return;
    const int e = idx[a];
    const int pos = offsets[e] + blockoff[size_t(e) * nblk + blockIdx.x] + lrank[a];
    perm[pos] = a;
    inv[a] = pos;
}

// ------------------------------------------------------------------------------------------ permute / combine
// xs[inv[t*k + j]] = x[t] for j < k: one wave per token reads the row once and scatters it to the
// token's k places in the expert-sorted order (reading by sorted position instead would fetch every
// token row k times, since a token's uses sit in k different groups).  d is a multiple of 8.
// The first MAX_K places sit in registers; a token with more uses looks the others up as it goes.
__global__ __launch_bounds__(256) void k_permute(const bf16_t* __restrict__ x, const int32_t* __restrict__ inv,
                                                 bf16_t* __restrict__ xs, int T, int d, int k)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int32_t* inv_t = inv + size_t(t) * k;
    int pos[MAX_K];
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) pos[j] = j < k ? inv_t[j] : 0;
    const u32x4* src = reinterpret_cast<const u32x4*>(x + size_t(t) * d);
    for (int c0 = 0; c0 < d / 8; c0 += 256) {
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = c0 + i * 64 + lane;
            if (c < d / 8) v[i] = src[c];
        }
        auto put = [&](int p) {
            u32x4* dst = reinterpret_cast<u32x4*>(xs + size_t(p) * d);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = c0 + i * 64 + lane;
                if (c < d / 8) dst[c] = v[i];
            }
        };
#pragma unroll
        for (int j = 0; j < MAX_K; ++j)
            if (j < k) put(pos[j]);
        for (int j = MAX_K; j < k; ++j) put(inv_t[j]);
    }
}

__global__ __launch_bounds__(256) void k_combine(const bf16_t* __restrict__ y, const int32_t* __restrict__ inv,
                                                 const float* __restrict__ topk_w, bf16_t* __restrict__ out,
                                                 int T, int d, int k)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int32_t* inv_t = inv + size_t(t) * k;
    const float* w_t = topk_w + size_t(t) * k;
    int pos[MAX_K];
    float w[MAX_K];
#pragma unroll
    for (int j = 0; j < MAX_K; ++j)
        if (j < k) { pos[j] = inv_t[j]; w[j] = w_t[j]; }
    for (int c = lane; c < d / 8; c += 64) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        auto add = [&](int p, float wj) {                  // j ascending: the summation order is fixed
            const u32x4 v = reinterpret_cast<const u32x4*>(y + size_t(p) * d)[c];
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] += wj * __uint_as_float(u[i] << 16);
                acc[2 * i + 1] += wj * __uint_as_float(u[i] & 0xffff0000u);
            }
        };
#pragma unroll
        for (int j = 0; j < MAX_K; ++j)
            if (j < k) add(pos[j], w[j]);
        for (int j = MAX_K; j < k; ++j) add(inv_t[j], w_t[j]);
        u32x4 o;
        o.x = pack_bf16x2(acc[0], acc[1]);
        o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]);
        o.w = pack_bf16x2(acc[6], acc[7]);
        reinterpret_cast<u32x4*>(out + size_t(t) * d)[c] = o;
    }
}

// ------------------------------------------------------------------------------------------ grouped GEMM
// Tile body: out[row0 .. row0+rows)[nb .. nb+TN) = act(in[rows][K] . We[n][K]^T), ML = live 16-row tiles.
//
// Operands go through LDS in K-chunks of 64.  Loading MFMA fragments straight from global memory
// makes every lane of a load touch its own 16 bytes of a different row, and the vector L1 then
// retires about one lane per clock (measured: ~16 B/clk per CU, which capped this kernel at 2 ms
// per layer).  Staged loads instead let 8 neighbouring lanes read one row's 128 contiguous bytes;
// the fragments are then cut out of LDS with ds_read_b128 (row pitch 144 bytes, conflict free).
// The next chunk is fetched into registers while the current one is multiplied: 40 KB per
// workgroup, two workgroups per CU.  (Tiles of 128 features with four workgroups per CU stream
// the second layer's 4 KB-pitched weight rows 15 % slower and are no faster elsewhere.)
constexpr int KC = 64;                 // K-chunk
constexpr int LDP = KC + 8;            // LDS row pitch in elements (144 bytes)

// gather != nullptr: the tile's input rows are not in[row0 ..] but rows of `in` picked through the
// grouping: row r of the tile is in[gather[row0 + r] / kdiv] (the token of that expert use), i.e. the
// stacking of the tokens happens inside the operand load and the permuted copy is never written.
template <bool RELU, int ML>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ in, const bf16_t* __restrict__ We,
                                          bf16_t* __restrict__ out, int row0, int rows, int nb, int N, int K,
                                          bf16_t* Ws, bf16_t* Xs, const int32_t* __restrict__ gather, int kdiv)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    constexpr int PARTS = KC / 8;                  // 16-byte pieces of one chunk row
    constexpr int RPP = 256 / PARTS;               // rows staged per pass of the workgroup
    constexpr int WPASS = TN / RPP, XPASS = TM / RPP;
    const int part = tid % PARTS, prow = tid / PARTS;
    // staging assignments: WPASS weight rows and up to XPASS activation rows per thread
    const bf16_t* wsrc[WPASS];
    const bf16_t* xsrc[XPASS];
#pragma unroll
    for (int i = 0; i < WPASS; ++i) wsrc[i] = We + size_t(min(nb + prow + i * RPP, N - 1)) * K + part * 8;
#pragma unroll
    for (int i = 0; i < XPASS; ++i) {
        const int r = row0 + min(prow + i * RPP, rows - 1);
        xsrc[i] = in + size_t(gather ? gather[r] / kdiv : r) * K + part * 8;
    }
    u32x4 wreg[WPASS], xreg[XPASS];
    auto fetch = [&](int kc) {
        const bool inside = kc * KC + part * 8 < K;   // K is a multiple of 8: the last chunk may be partly empty
#pragma unroll
        for (int i = 0; i < WPASS; ++i)
            wreg[i] = inside ? *reinterpret_cast<const u32x4*>(wsrc[i] + kc * KC) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < XPASS; ++i)
            if (i * RPP < ML * 16)                    // only rows of live 16-row sub-tiles
                xreg[i] = inside ? *reinterpret_cast<const u32x4*>(xsrc[i] + kc * KC) : u32x4{0u, 0u, 0u, 0u};
    };
    const int nchunk = (K + KC - 1) / KC;
    // one K-chunk through LDS: registers -> LDS, barrier, prefetch of the next chunk, multiply, barrier
    auto chunk_loop = [&](auto&& multiply) {
        fetch(0);
        for (int kc = 0; kc < nchunk; ++kc) {
#pragma unroll
            for (int i = 0; i < WPASS; ++i)
                *reinterpret_cast<u32x4*>(Ws + (prow + i * RPP) * LDP + part * 8) = wreg[i];
#pragma unroll
            for (int i = 0; i < XPASS; ++i)
                if (i * RPP < ML * 16) *reinterpret_cast<u32x4*>(Xs + (prow + i * RPP) * LDP + part * 8) = xreg[i];
            __syncthreads();
            if (kc + 1 < nchunk) fetch(kc + 1);
            multiply();
            __syncthreads();
        }
    };
    const int n0 = nb + wave * (TN / 4);          // first feature of this wave
    auto store4 = [&](int lr, int n, float v0, float v1, float v2, float v3) {
        if (lr >= rows || n >= N) return;
        u32x2 pk;
        pk.x = pack_bf16x2(v0, v1);
        pk.y = pack_bf16x2(v2, v3);
        if (RELU) { pk.x = relu_bf16x2(pk.x); pk.y = relu_bf16x2(pk.y); }
        *reinterpret_cast<u32x2*>(out + size_t(row0 + lr) * N + n) = pk;
    };
    if constexpr (ML == 4) {
        // all four 16-row sub-tiles live: 32x32x16 MFMAs (the faster bf16 shape), 2 x 2 tiles per wave
        static_assert(TN == 256, "two 32-feature tiles per wave");
        const int q = lane & 31, hk = lane >> 5;
        f32x16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        chunk_loop([&] {
#pragma unroll
            for (int ks = 0; ks < KC / 16; ++ks) {
                bf16x8 wf[2], xf[2];
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    wf[a] = *reinterpret_cast<const bf16x8*>(Ws + (wave * 64 + a * 32 + q) * LDP + ks * 16 + hk * 8);
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    xf[b] = *reinterpret_cast<const bf16x8*>(Xs + (b * 32 + q) * LDP + ks * 16 + hk * 8);
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
            }
        });
        // lane holds row b*32 + q, features n0 + a*32 + 8j + 4hk .. +3 in acc[a][b][4j .. 4j+3]
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    store4(b * 32 + q, n0 + a * 32 + 8 * j + 4 * hk, acc[a][b][4 * j], acc[a][b][4 * j + 1],
                           acc[a][b][4 * j + 2], acc[a][b][4 * j + 3]);
    } else {
        f32x4 acc[ML][NTW];
#pragma unroll
        for (int mt = 0; mt < ML; ++mt)
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) acc[mt][nt] = f32x4{0, 0, 0, 0};
        chunk_loop([&] {
#pragma unroll
            for (int kk = 0; kk < KC / 32; ++kk) {
                bf16x8 wf[NTW], xf[ML];
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt)
                    wf[nt] = *reinterpret_cast<const bf16x8*>(Ws + (wave * (TN / 4) + nt * 16 + r) * LDP + kk * 32 + g * 8);
#pragma unroll
                for (int mt = 0; mt < ML; ++mt)
                    xf[mt] = *reinterpret_cast<const bf16x8*>(Xs + (mt * 16 + r) * LDP + kk * 32 + g * 8);
#pragma unroll
                for (int mt = 0; mt < ML; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt], xf[mt], acc[mt][nt], 0, 0, 0);
            }
        });
        // lane holds features n0 + nt*16 + g*4 .. +3 of row mt*16 + r
#pragma unroll
        for (int mt = 0; mt < ML; ++mt)
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt)
                store4(mt * 16 + r, n0 + nt * 16 + g * 4, acc[mt][nt].x, acc[mt][nt].y, acc[mt][nt].z, acc[mt][nt].w);
    }
}

// out[row][n] = act( sum_k in[row][k] * W[e][n][k] ) for the rows of expert e.
// One workgroup = one (row tile of <= 64 rows inside one group, 256 output features) pair; a group's
// tiles are found from tile_start (prefix sum of ceil(count/64)), so ragged and empty groups cost
// nothing beyond their real rows.  4 waves split the 256 features; only the live 16-row sub-tiles
// are multiplied.  N must be a multiple of 4 (it is: d and h are multiples of 8).
template <bool RELU>
__global__ __launch_bounds__(256) void k_grouped_gemm(const bf16_t* __restrict__ in, const bf16_t* __restrict__ W,
                                                      bf16_t* __restrict__ out, const int32_t* __restrict__ offsets,
                                                      const int32_t* __restrict__ tile_start, int E, int N, int K,
                                                      int n_tiles_n, int chunk, const int32_t* __restrict__ gather, int kdiv)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ws[TN * LDP];
    __shared__ __attribute__((aligned(16))) bf16_t Xs[TM * LDP];
    // Tiles are numbered expert by expert; inside an expert, row tiles are taken in groups of MG, and
    // inside a group the row tiles that share one feature tile are adjacent (feature tile outer, row
    // tile inner), so a weight tile is fetched from HBM once and then found in L2 by the other row
    // tiles of its group.  Consecutive workgroup ids land on different XCDs (8 of them, each with
    // its own L2), so the numbering is dealt to the XCDs in runs of `chunk` tiles: everything that
    // shares weights or activation rows stays behind one L2.
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const long long lin = (long long)(j / chunk * 8 + xcd) * chunk + j % chunk;
    if (lin >= (long long)tile_start[E] * n_tiles_n) return;
    const int lin_m = int(lin / n_tiles_n);
    int lo = 0, hi = E;                          // largest e with tile_start[e] <= lin_m
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_start[mid] <= lin_m) lo = mid; else hi = mid;
    }
    const int e = lo;
    const int mt_e = tile_start[e + 1] - tile_start[e];
    const int i = int(lin - (long long)tile_start[e] * n_tiles_n);   // tile of this expert, 0 .. mt_e * n_tiles_n
    const int mg = i / (MG * n_tiles_n);
    const int rem = i - mg * MG * n_tiles_n;
    const int gsize = min(MG, mt_e - mg * MG);
    const int ntile = rem / gsize;
    const int mtile = mg * MG + rem % gsize;
    const int row0 = offsets[e] + mtile * TM;
    const int rows = min(TM, offsets[e + 1] - row0);
    const int mlive = (rows + 15) >> 4;
    const bf16_t* We = W + size_t(e) * N * K;
    const int nb = ntile * TN;
    if (mlive <= 1) gemm_tile<RELU, 1>(in, We, out, row0, rows, nb, N, K, Ws, Xs, gather, kdiv);
    else if (mlive == 2) gemm_tile<RELU, 2>(in, We, out, row0, rows, nb, N, K, Ws, Xs, gather, kdiv);
    else gemm_tile<RELU, 4>(in, We, out, row0, rows, nb, N, K, Ws, Xs, gather, kdiv);
}

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

struct Layout {
    size_t logits, topk_idx, topk_w, counts, offsets, tile_start, perm, inv, lrank, blockcnt, xs, hid, y, total;
    int nblk;
};

Layout layout(const moe_shape* s)
{
    Layout L;
    const size_t T = size_t(s->T), E = size_t(s->E), A = T * size_t(s->k);
    L.nblk = int((A + SORT_BLOCK - 1) / SORT_BLOCK);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(std::max<size_t>(bytes, 4)); return at; };
    L.logits = take(T * E * 4);
    L.topk_idx = take(A * 4);
    L.topk_w = take(A * 4);
    L.counts = take(E * 4);
    L.offsets = take((E + 1) * 4);
    L.tile_start = take((E + 1) * 4);
    L.perm = take(A * 4);
    L.inv = take(A * 4);
    L.lrank = take(A * 4);
    L.blockcnt = take(E * size_t(std::max(L.nblk, 1)) * 4);
    L.xs = take(A * size_t(s->d) * 2);
    L.hid = take(A * size_t(s->h) * 2);
    L.y = take(A * size_t(s->d) * 2);
    L.total = o;
    return L;
}

int check_shape(const moe_shape* s, const char* who)
{
    if (!s) return fail(DYNB_E_INVAL, std::string(who) + ": NULL shape");
    if (size_t(s->T) > size_t(65535) * 64) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": more than 4194240 tokens");
    if (s->T < 0 || s->d <= 0 || s->h <= 0 || s->E <= 0 || s->k <= 0)
        return fail(DYNB_E_INVAL, std::string(who) + ": sizes must be positive");
    if (s->k > s->E) return fail(DYNB_E_INVAL, std::string(who) + ": k > E");
    if (s->d % 8 || s->h % 8)
        return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": d and h must be multiples of 8 (rows are moved in 16-byte pieces)");
    if (s->dtype != DYNB_BF16) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": only bf16");
    if (s->flags & ~uint32_t(MOE_SEPARATE_PERMUTE)) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": unknown flag bits");
    if (size_t(s->T) * size_t(s->k) >= (size_t(1) << 30) || size_t(s->T) * size_t(s->E) >= (size_t(1) << 40))
        return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": too many expert uses");
    // the grouped expert layers launch one workgroup per (row tile, feature tile): at most ceil(A/TM) + E row tiles
    const long long max_mtiles = ((long long)s->T * s->k + TM - 1) / TM + s->E;
    const long long nt = (std::max(s->h, s->d) + TN - 1) / TN;
    if (max_mtiles * nt + 8ll * XCD_CHUNK >= (1ll << 31)) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": grid too large");
    return DYNB_OK;
}

}  // namespace

extern "C" size_t moe_workspace_bytes(const moe_shape* s)
{
    if (check_shape(s, "moe_workspace_bytes") != DYNB_OK) return 0;
    return std::max<size_t>(layout(s).total, 256);
}

__global__ void k_unit_group(int32_t* p)      // offsets {0,1} and tile table {0,1} of a one-row group
{
    if (threadIdx.x < 4) p[threadIdx.x] = threadIdx.x & 1;
}

// naive_stride = 0: batched layer.  naive_stride >= 1: the expert stage is run one use at a time
// (every naive_stride-th use), which needs the group sizes on the host.
static int moe_run(const moe_shape* s, const void* x, const void* Wg, const void* Wn, const float* noise,
                   const void* W1, const void* W2, void* out, const moe_aux* aux, void* workspace,
                   size_t workspace_bytes, void* stream, int naive_stride)
{
    int rc = check_shape(s, "moe_forward");
    if (rc != DYNB_OK) return rc;
    if (s->T == 0) return DYNB_OK;
    if (!x || !Wg || !W1 || !W2 || !out || !workspace) return fail(DYNB_E_INVAL, "moe_forward: NULL argument");
    if (noise && !Wn) return fail(DYNB_E_INVAL, "moe_forward: noise given without Wn");
    const Layout L = layout(s);
    if (workspace_bytes < L.total) return fail(DYNB_E_WORKSPACE, "moe_forward: workspace too small");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(DYNB_E_INVAL, "moe_forward: workspace not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const int T = s->T, d = s->d, h = s->h, E = s->E, k = s->k, A = T * k;

    float* logits = (aux && aux->logits) ? aux->logits : reinterpret_cast<float*>(ws + L.logits);
    int32_t* topk_idx = (aux && aux->topk_idx) ? aux->topk_idx : reinterpret_cast<int32_t*>(ws + L.topk_idx);
    float* topk_w = (aux && aux->topk_w) ? aux->topk_w : reinterpret_cast<float*>(ws + L.topk_w);
    int32_t* counts = (aux && aux->counts) ? aux->counts : reinterpret_cast<int32_t*>(ws + L.counts);
    int32_t* offsets = (aux && aux->offsets) ? aux->offsets : reinterpret_cast<int32_t*>(ws + L.offsets);
    int32_t* perm = (aux && aux->perm) ? aux->perm : reinterpret_cast<int32_t*>(ws + L.perm);
    int32_t* inv = (aux && aux->inv) ? aux->inv : reinterpret_cast<int32_t*>(ws + L.inv);
    int32_t* tile_start = reinterpret_cast<int32_t*>(ws + L.tile_start);
    int32_t* lrank = reinterpret_cast<int32_t*>(ws + L.lrank);
    int32_t* blockcnt = reinterpret_cast<int32_t*>(ws + L.blockcnt);
    bf16_t* xs = reinterpret_cast<bf16_t*>(ws + L.xs);
    bf16_t* hid = reinterpret_cast<bf16_t*>(ws + L.hid);
    bf16_t* y = reinterpret_cast<bf16_t*>(ws + L.y);
    const bf16_t* xb = static_cast<const bf16_t*>(x);

    const bool timed = dynb::timing_on();
    if (timed) dynb::timing_begin(st);
    // m1 gate
    // whole tiles of 256 tokens go to k_gate_big where the expert and model widths allow it, the tokens behind the
    // last whole tile (and every other shape) to k_gate
    const int T_big = (E % GB_EXP == 0 && d % GKC == 0 && d >= 4 * GKC && size_t(GB_TOK) * size_t(std::max(E, d)) < (size_t(1) << 30))
                          ? T / GB_TOK * GB_TOK : 0;
    if (T_big > 0) {
        static std::atomic<uint64_t> attr_set{0};             // one bit per device: LDS beyond 64 KB
        int dev = 0;
        HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
        if (!(attr_set.load() >> (dev & 63) & 1)) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gate_big<true>), hipFuncAttributeMaxDynamicSharedMemorySize, GB_LDS_BYTES),
                    "hipFuncSetAttribute(k_gate_big)");
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gate_big<false>), hipFuncAttributeMaxDynamicSharedMemorySize, GB_LDS_BYTES),
                    "hipFuncSetAttribute(k_gate_big)");
            attr_set.fetch_or(uint64_t(1) << (dev & 63));
        }
        const int ntt = T_big / GB_TOK, net = E / GB_EXP, per_die = (ntt + 7) / 8;
        const dim3 grid(unsigned(8 * per_die * net));
        if (noise)
            hipLaunchKernelGGL((k_gate_big<true>), grid, dim3(256), GB_LDS_BYTES, st, xb, static_cast<const bf16_t*>(Wg),
                               static_cast<const bf16_t*>(Wn), noise, logits, T_big, d, E, ntt, net, per_die);
        else
            hipLaunchKernelGGL((k_gate_big<false>), grid, dim3(256), GB_LDS_BYTES, st, xb, static_cast<const bf16_t*>(Wg),
                               static_cast<const bf16_t*>(Wn), noise, logits, T_big, d, E, ntt, net, per_die);
    }
    if (T > T_big)
        hipLaunchKernelGGL(k_gate, dim3((E + 63) / 64, (T - T_big + 63) / 64), dim3(256), 0, st, xb + size_t(T_big) * d,
                           static_cast<const bf16_t*>(Wg), static_cast<const bf16_t*>(Wn), noise ? noise + size_t(T_big) * E : nullptr,
                           logits + size_t(T_big) * E, T - T_big, d, E);
    if (timed) dynb::timing_mark(st, dynb::ST_GATE, 0);
    // m2 top-k + softmax
    const dim3 tk_grid((T + 3) / 4), tk_block(256);
    if (k <= MAX_K && E <= 4 * 64)
        hipLaunchKernelGGL((k_topk_small<4>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else if (k <= MAX_K && E <= 16 * 64)
        hipLaunchKernelGGL((k_topk_small<16>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else if (k <= MAX_K && E <= 32 * 64)
        hipLaunchKernelGGL((k_topk_small<32>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else if (E <= 4 * 64)
        hipLaunchKernelGGL((k_topk<4>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else if (E <= 16 * 64)
        hipLaunchKernelGGL((k_topk<16>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else if (E <= 32 * 64)
        hipLaunchKernelGGL((k_topk<32>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    else
        hipLaunchKernelGGL((k_topk<0>), tk_grid, tk_block, 0, st, logits, topk_idx, topk_w, T, E, k);
    if (timed) dynb::timing_mark(st, dynb::ST_TOPK, 0);
    // m3 stable counting sort
    const size_t nbc = size_t(E) * L.nblk;
    hipLaunchKernelGGL(k_zero_i32, dim3(unsigned(std::min<size_t>((nbc + 255) / 256, 2048))), dim3(256), 0, st, blockcnt, nbc);
    hipLaunchKernelGGL(k_rank_blocks, dim3(L.nblk), dim3(SORT_BLOCK), 0, st, topk_idx, lrank, blockcnt, A, L.nblk);
    hipLaunchKernelGGL(k_scan_blocks, dim3((E + 3) / 4), dim3(256), 0, st, blockcnt, counts, E, L.nblk);
    hipLaunchKernelGGL(k_offsets, dim3(1), dim3(OFFS_THREADS), 0, st, counts, offsets, tile_start, E);
    hipLaunchKernelGGL(k_place, dim3(L.nblk), dim3(SORT_BLOCK), 0, st, topk_idx, lrank, blockcnt, offsets, perm, inv, A, L.nblk);
    if (timed) dynb::timing_mark(st, dynb::ST_SORT, 0);
    // m4 permute: as a kernel of its own (MOE_SEPARATE_PERMUTE, and for the per-use loop), else inside the
    // first expert layer's operand load, which reads token perm[pos] / k for sorted position pos
    const bool fused_permute = !(s->flags & MOE_SEPARATE_PERMUTE) && naive_stride <= 0;
    if (!fused_permute) hipLaunchKernelGGL(k_permute, dim3((T + 3) / 4), dim3(256), 0, st, xb, inv, xs, T, d, k);
    if (timed) dynb::timing_mark(st, dynb::ST_PERMUTE, 0);
    // m5 grouped expert FFN: at most ceil(A/TM) + E row tiles exist
    const long long max_mtiles = (long long)(A + TM - 1) / TM + E;
    const int nt1 = (h + TN - 1) / TN, nt2 = (d + TN - 1) / TN;
    if (naive_stride <= 0) {
        const long long span = 8ll * XCD_CHUNK;
        hipLaunchKernelGGL((k_grouped_gemm<true>), dim3(unsigned((max_mtiles * nt1 + span - 1) / span * span)), dim3(256), 0, st,
                           fused_permute ? xb : xs, static_cast<const bf16_t*>(W1), hid, offsets, tile_start, E, h, d, nt1,
                           XCD_CHUNK, fused_permute ? perm : nullptr, k);
        if (timed) dynb::timing_mark(st, dynb::ST_FFN1, 0);
        hipLaunchKernelGGL((k_grouped_gemm<false>), dim3(unsigned((max_mtiles * nt2 + span - 1) / span * span)), dim3(256), 0, st,
                           hid, static_cast<const bf16_t*>(W2), y, offsets, tile_start, E, d, h, nt2, XCD_CHUNK, nullptr, 1);
        if (timed) dynb::timing_mark(st, dynb::ST_FFN2, 0);
    } else {
        // the paper's naive version: loop over the k*b expert uses, one expert call (two layers) per use
        std::vector<int32_t> off(size_t(E) + 1);
        int32_t* unit = lrank;                                // free again after k_place
        hipLaunchKernelGGL(k_unit_group, dim3(1), dim3(64), 0, st, unit);
        HIP_TRY(hipMemcpyAsync(off.data(), offsets, off.size() * sizeof(int32_t), hipMemcpyDeviceToHost, st), "moe_forward_naive");
        HIP_TRY(hipStreamSynchronize(st), "moe_forward_naive");
        const bf16_t* w1 = static_cast<const bf16_t*>(W1);
        const bf16_t* w2 = static_cast<const bf16_t*>(W2);
        for (int e = 0; e < E; ++e)
            for (int pos = off[e]; pos < off[e + 1]; ++pos) {
                if (pos % naive_stride) continue;
                hipLaunchKernelGGL((k_grouped_gemm<true>), dim3((nt1 + 7) / 8 * 8), dim3(256), 0, st, xs + size_t(pos) * d,
                                   w1 + size_t(e) * h * d, hid + size_t(pos) * h, unit, unit + 2, 1, h, d, nt1, 1, nullptr, 1);
                hipLaunchKernelGGL((k_grouped_gemm<false>), dim3((nt2 + 7) / 8 * 8), dim3(256), 0, st, hid + size_t(pos) * h,
                                   w2 + size_t(e) * d * h, y + size_t(pos) * d, unit, unit + 2, 1, d, h, nt2, 1, nullptr, 1);
            }
        if (timed) { dynb::timing_mark(st, dynb::ST_FFN1, 0); dynb::timing_mark(st, dynb::ST_FFN2, 0); }
    }
    // m6 combine
    hipLaunchKernelGGL(k_combine, dim3((T + 3) / 4), dim3(256), 0, st, y, inv, topk_w, static_cast<bf16_t*>(out), T, d, k);
    if (timed) dynb::timing_mark(st, dynb::ST_COMBINE, 0);
    HIP_TRY(hipGetLastError(), "moe_forward");
    return DYNB_OK;
}

extern "C" int moe_forward(const moe_shape* s, const void* x, const void* Wg, const void* Wn, const float* noise,
                           const void* W1, const void* W2, void* out, const moe_aux* aux, void* workspace,
                           size_t workspace_bytes, void* stream)
{
    return moe_run(s, x, Wg, Wn, noise, W1, W2, out, aux, workspace, workspace_bytes, stream, 0);
}

// ------------------------------------------------------------------------------------------
// Entry point for callers that cannot allocate device memory.  The routing tables and the
// xs / hid / y buffers that moe_forward keeps in its caller-provided workspace live in a device
// array that is part of the library's code object; every GPU holds its own copy at its own address.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current GPU.  In host code the array's name is only a
// stand-in for the symbol, so the address is asked for once per device and kept.
static int static_scratch_ptr(void** out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void* ptr_of[MAX_DEVICES] = {};
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev), "moe_forward_static(hipGetDevice)");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(DYNB_E_UNSUPPORTED, "moe_forward_static: device ordinal beyond 63");
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "moe_forward_static(hipGetSymbolAddress)");
        if (!p) return fail(DYNB_E_HIP, "moe_forward_static: no device address for the scratch array");
        ptr_of[dev] = p;
    }
    *out = ptr_of[dev];
    return DYNB_OK;
}

extern "C" int moe_forward_static(const moe_shape* s, const void* x, const void* Wg, const void* Wn, const float* noise,
                                  const void* W1, const void* W2, void* out, const moe_aux* aux, void* stream)
{
    int rc = check_shape(s, "moe_forward_static");
    if (rc != DYNB_OK) return rc;
    const size_t need = layout(s).total;
    if (need > size_t(MOE_STATIC_SCRATCH_BYTES))
        return fail(DYNB_E_WORKSPACE, "moe_forward_static: this shape needs " + std::to_string(need) +
                                          " bytes of scratch memory, the built-in array holds " +
                                          std::to_string(size_t(MOE_STATIC_SCRATCH_BYTES)) + "; use moe_forward");
    void* ws = nullptr;
    rc = static_scratch_ptr(&ws);
    if (rc != DYNB_OK) return rc;
    // every buffer of the layout is written before it is read, and the one table that must start
    // at zero (blockcnt) is cleared by a fill kernel inside the layer: the previous call's contents do not matter
    return moe_run(s, x, Wg, Wn, noise, W1, W2, out, aux, ws, size_t(MOE_STATIC_SCRATCH_BYTES), stream, 0);
}

extern "C" int moe_forward_naive(const moe_shape* s, const void* x, const void* Wg, const void* Wn, const float* noise,
                                 const void* W1, const void* W2, void* out, const moe_aux* aux, void* workspace,
                                 size_t workspace_bytes, void* stream, int32_t use_stride)
{
    if (use_stride < 1) return fail(DYNB_E_INVAL, "moe_forward_naive: use_stride must be >= 1");
    return moe_run(s, x, Wg, Wn, noise, W1, W2, out, aux, workspace, workspace_bytes, stream, use_stride);
}
