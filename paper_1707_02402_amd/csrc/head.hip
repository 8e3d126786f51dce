// Classifier head on the root maps of a batch (paper: Background / Visual Reasoning Programs: the executed
// program's output passes through one convolutional and two fully connected layers and a softmax over the
// answers).  The paper fixes neither sizes nor the kernel shape; the reading taken here is a 1x1 convolution
// C -> Cc with ReLU, the map flattened in [H][W][Cc] order, a fully connected layer to F units with ReLU, a
// fully connected layer to A answers, softmax.
//
// All three layers are the same contraction, out[m][n] = act(sum_k a[m][k] * w[n][k] + bias[n]), with both
// operands stored row by row along k:
//   conv 1x1   a = root maps   [B*H*W][C]      w = wc  [Cc][C]
//   fc 1       a = conv output [B][H*W*Cc]     w = wf1 [F][H*W*Cc]
//   fc 2       a = fc 1 output [B][F]          w = wf2 [A][F]
// bf16 operands whose k extent is a multiple of 8 run on 32x32x16 MFMAs from LDS-staged 64 x 64 tiles;
// everything else (fp32 storage, odd k) runs a plain FMA tile kernel.  A layer with few output tiles and a long
// k (fc 1: 16 tiles, k = 6272) is cut along k into `splits` slices that are summed afterwards in slice order, so
// the result does not depend on how the workgroups were scheduled.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "device_utils.h"
#include "plan_internal.h"

using dynb::fail;

#define HIP_TRY(expr, what)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(DYNB_E_HIP, std::string(what) + ": " + hipGetErrorString(e_));        \
    } while (0)

namespace {

constexpr int HT = 64;            // tile side (rows of a and rows of w per workgroup)
constexpr int HKC = 64;           // k chunk of the MFMA kernel
constexpr int HLDP = HKC + 8;     // LDS row pitch in elements (144 bytes: conflict-free 16-byte reads)

struct GemmArgs {
    const void* a;       // [M][K]
    const void* w;       // [N][K]
    float* part;         // [splits][M][N] partial sums (fp32)
    int M, N, K;
    int kslice;          // k extent of one split (a multiple of the kernel's chunk)
};

// part[z][m][n] = sum over the z-th k slice of a[m][k] * w[n][k]; bf16 operands, K a multiple of 8.
__global__ __launch_bounds__(256) void k_head_gemm_mfma(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) bf16_t As[HT * HLDP];
    __shared__ __attribute__((aligned(16))) bf16_t Ws[HT * HLDP];
    const bf16_t* a = static_cast<const bf16_t*>(g.a);
    const bf16_t* w = static_cast<const bf16_t*>(g.w);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int m0 = blockIdx.y * HT, n0 = blockIdx.x * HT;
    const int k_lo = blockIdx.z * g.kslice, k_hi = min(g.K, k_lo + g.kslice);
    const int part8 = tid & 7, srow = tid >> 3;           // staging: 32 rows x 8 pieces of 16 bytes per pass
    const bf16_t* asrc[2];
    const bf16_t* wsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        asrc[i] = a + size_t(min(m0 + srow + i * 32, g.M - 1)) * g.K + part8 * 8;
        wsrc[i] = w + size_t(min(n0 + srow + i * 32, g.N - 1)) * g.K + part8 * 8;
    }
    u32x4 areg[2], wreg[2];
    auto fetch = [&](int k) {
        const bool inside = k + part8 * 8 < k_hi;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            areg[i] = inside ? *reinterpret_cast<const u32x4*>(asrc[i] + k) : u32x4{0u, 0u, 0u, 0u};
            wreg[i] = inside ? *reinterpret_cast<const u32x4*>(wsrc[i] + k) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    // 4 waves = 2 halves of the a rows x 2 halves of the w rows, one 32 x 32 tile each
    const int q = lane & 31, hk = lane >> 5, mh = wave & 1, nh = wave >> 1;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    fetch(k_lo);
    for (int k = k_lo; k < k_hi; k += HKC) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<u32x4*>(As + (srow + i * 32) * HLDP + part8 * 8) = areg[i];
            *reinterpret_cast<u32x4*>(Ws + (srow + i * 32) * HLDP + part8 * 8) = wreg[i];
        }
        __syncthreads();
        if (k + HKC < k_hi) fetch(k + HKC);
#pragma unroll
        for (int ks = 0; ks < HKC / 16; ++ks) {
            const bf16x8 af = *reinterpret_cast<const bf16x8*>(As + (mh * 32 + q) * HLDP + ks * 16 + hk * 8);
            const bf16x8 wf = *reinterpret_cast<const bf16x8*>(Ws + (nh * 32 + q) * HLDP + ks * 16 + hk * 8);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, wf, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // lane holds column n0 + nh*32 + q, rows m0 + mh*32 + 8*(i/4) + 4*hk + i%4 in element i
    const int n = n0 + nh * 32 + q;
    if (n >= g.N) return;
    float* out = g.part + size_t(blockIdx.z) * g.M * g.N;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int m = m0 + mh * 32 + 8 * (i / 4) + 4 * hk + (i % 4);
        if (m < g.M) out[size_t(m) * g.N + n] = acc[i];
    }
}

// The same contraction with plain fp32 FMAs for any storage type and any K: 64 x 64 tile, 4 x 4 outputs per thread.
template <typename T>
__global__ __launch_bounds__(256) void k_head_gemm_fma(GemmArgs g)
{
    constexpr int KC = 16;
    __shared__ float As[KC][HT + 1];
    __shared__ float Ws[KC][HT + 1];
    const T* a = static_cast<const T*>(g.a);
    const T* w = static_cast<const T*>(g.w);
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * HT, n0 = blockIdx.x * HT;
    const int k_lo = blockIdx.z * g.kslice, k_hi = min(g.K, k_lo + g.kslice);
    const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k = k_lo; k < k_hi; k += KC) {
        for (int e = tid; e < HT * KC; e += 256) {
            const int r = e / KC, kk = e % KC;
            const bool kin = k + kk < k_hi;
            As[kk][r] = (kin && m0 + r < g.M) ? load_f32(a + size_t(m0 + r) * g.K + k + kk) : 0.f;
            Ws[kk][r] = (kin && n0 + r < g.N) ? load_f32(w + size_t(n0 + r) * g.K + k + kk) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            float av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[kk][tm + i]; wv[i] = Ws[kk][tn + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * wv[j];
        }
        __syncthreads();
    }
    float* out = g.part + size_t(blockIdx.z) * g.M * g.N;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (m0 + tm + i < g.M && n0 + tn + j < g.N) out[size_t(m0 + tm + i) * g.N + n0 + tn + j] = acc[i][j];
}

// out[m][n] = act(bias[n] + part[0][m][n] + part[1][m][n] + ...), slices in ascending order
template <typename TO, bool RELU>
__global__ void k_head_finish(const float* __restrict__ part, const float* __restrict__ bias, TO* __restrict__ out,
                              size_t MN, int N, int splits)
{
    for (size_t e = size_t(blockIdx.x) * blockDim.x + threadIdx.x; e < MN; e += size_t(gridDim.x) * blockDim.x) {
        float v = bias ? bias[e % N] : 0.f;
        for (int z = 0; z < splits; ++z) v += part[size_t(z) * MN + e];
        if (RELU) v = fmaxf(v, 0.f);
        store_f32(out + e, v);
    }
}

// one wave per example: probs = softmax(logits)
__global__ __launch_bounds__(256) void k_head_softmax(const float* __restrict__ logits, float* __restrict__ probs, int B, int A)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= B) return;
    const float* row = logits + size_t(i) * A;
    float mx = -INFINITY;
    for (int a = lane; a < A; a += 64) mx = fmaxf(mx, row[a]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float den = 0.f;
    for (int a = lane; a < A; a += 64) den += expf(row[a] - mx);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
    for (int a = lane; a < A; a += 64) probs[size_t(i) * A + a] = expf(row[a] - mx) / den;
}

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
size_t elt(int dtype) { return dtype == DYNB_BF16 ? 2 : 4; }

// k slices of a layer: enough workgroups to fill the chip, never more than the chunks there are
int splits_for(int M, int N, int K)
{
    const long long tiles = (long long)((M + HT - 1) / HT) * ((N + HT - 1) / HT);
    const int chunks = (K + HKC - 1) / HKC;
    if (tiles >= 256 || chunks <= 1) return 1;
    return int(std::max<long long>(1, std::min<long long>(chunks, std::min<long long>(64, (512 + tiles - 1) / tiles))));
}

struct HeadLayout {
    size_t z, h1, logits, part, total;
    int s1, s2, s3;
};

HeadLayout head_layout(const dynb_head_shape* s, int32_t B)
{
    HeadLayout L;
    const size_t P = size_t(s->H) * s->W, M1 = size_t(B) * P;
    L.s1 = splits_for(int(M1), s->Cc, s->C);
    L.s2 = splits_for(B, s->F, int(P * s->Cc));
    L.s3 = splits_for(B, s->n_answers, s->F);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(std::max<size_t>(bytes, 4)); return at; };
    L.z = take(M1 * s->Cc * elt(s->dtype));
    L.h1 = take(size_t(B) * s->F * elt(s->dtype));
    L.logits = take(size_t(B) * s->n_answers * 4);
    L.part = take(4 * std::max({size_t(L.s1) * M1 * s->Cc, size_t(L.s2) * B * s->F, size_t(L.s3) * B * s->n_answers}));
    L.total = o;
    return L;
}

int check_head(const dynb_head_shape* s, int32_t B, const char* who)
{
    if (!s) return fail(DYNB_E_INVAL, std::string(who) + ": NULL shape");
    if (B < 0 || s->C <= 0 || s->H <= 0 || s->W <= 0 || s->Cc <= 0 || s->F <= 0 || s->n_answers <= 0)
        return fail(DYNB_E_INVAL, std::string(who) + ": sizes must be positive");
    if (s->dtype != DYNB_F32 && s->dtype != DYNB_BF16) return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": unknown dtype");
    const unsigned long long big = 1ull << 31;
    if ((unsigned long long)B * s->H * s->W >= big || (unsigned long long)s->H * s->W * s->Cc >= big ||
        (unsigned long long)B * s->H * s->W * std::max(s->C, s->Cc) >= (1ull << 40))
        return fail(DYNB_E_UNSUPPORTED, std::string(who) + ": batch too large");
    return DYNB_OK;
}

template <typename TO, bool RELU>
void launch_layer(int dtype, const void* a, const void* w, const float* bias, TO* out, float* part, int M, int N, int K,
                  int splits, hipStream_t st)
{
    GemmArgs g{a, w, part, M, N, K, 0};
    const int chunks = (K + HKC - 1) / HKC;
    g.kslice = (chunks + splits - 1) / splits * HKC;
    const dim3 grid(unsigned((N + HT - 1) / HT), unsigned((M + HT - 1) / HT), unsigned((K + g.kslice - 1) / g.kslice));
    if (dtype == DYNB_BF16 && K % 8 == 0) hipLaunchKernelGGL(k_head_gemm_mfma, grid, dim3(256), 0, st, g);
    else if (dtype == DYNB_BF16) hipLaunchKernelGGL((k_head_gemm_fma<bf16_t>), grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL((k_head_gemm_fma<float>), grid, dim3(256), 0, st, g);
    const size_t MN = size_t(M) * N;
    hipLaunchKernelGGL((k_head_finish<TO, RELU>), dim3(unsigned(std::min<size_t>((MN + 255) / 256, 4096))), dim3(256), 0, st,
                       part, bias, out, MN, N, int(grid.z));
}

}  // namespace

extern "C" size_t dynbatch_classify_workspace_bytes(const dynb_head_shape* s, int32_t B)
{
    if (check_head(s, B, "dynbatch_classify_workspace_bytes") != DYNB_OK) return 0;
    return std::max<size_t>(head_layout(s, std::max(B, 1)).total, 256);
}

extern "C" int dynbatch_classify(const dynb_head_shape* s, const dynb_head_weights* w, const void* roots, int32_t B,
                                 float* probs, float* logits_out, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_head(s, B, "dynbatch_classify");
    if (rc != DYNB_OK) return rc;
    if (B == 0) return DYNB_OK;
    if (!w || !roots || !probs || !workspace) return fail(DYNB_E_INVAL, "dynbatch_classify: NULL argument");
    if (!w->wc || !w->wf1 || !w->wf2) return fail(DYNB_E_INVAL, "dynbatch_classify: a weight tensor is missing");
    const HeadLayout L = head_layout(s, B);
    if (workspace_bytes < L.total) return fail(DYNB_E_WORKSPACE, "dynbatch_classify: workspace too small");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(DYNB_E_INVAL, "dynbatch_classify: workspace not 256-byte aligned");
    if (s->dtype == DYNB_BF16 && ((reinterpret_cast<uintptr_t>(roots) | reinterpret_cast<uintptr_t>(w->wc) |
                                   reinterpret_cast<uintptr_t>(w->wf1) | reinterpret_cast<uintptr_t>(w->wf2)) & 15))
        return fail(DYNB_E_INVAL, "dynbatch_classify: bf16 tensors must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const int P = s->H * s->W, M1 = B * P, J = P * s->Cc;
    float* part = reinterpret_cast<float*>(ws + L.part);
    float* logits = logits_out ? logits_out : reinterpret_cast<float*>(ws + L.logits);
    if (s->dtype == DYNB_BF16) {
        bf16_t* z = reinterpret_cast<bf16_t*>(ws + L.z);
        bf16_t* h1 = reinterpret_cast<bf16_t*>(ws + L.h1);
        launch_layer<bf16_t, true>(s->dtype, roots, w->wc, w->bc, z, part, M1, s->Cc, s->C, L.s1, st);
        launch_layer<bf16_t, true>(s->dtype, z, w->wf1, w->bf1, h1, part, B, s->F, J, L.s2, st);
        launch_layer<float, false>(s->dtype, h1, w->wf2, w->bf2, logits, part, B, s->n_answers, s->F, L.s3, st);
    } else {
        float* z = reinterpret_cast<float*>(ws + L.z);
        float* h1 = reinterpret_cast<float*>(ws + L.h1);
        launch_layer<float, true>(s->dtype, roots, w->wc, w->bc, z, part, M1, s->Cc, s->C, L.s1, st);
        launch_layer<float, true>(s->dtype, z, w->wf1, w->bf1, h1, part, B, s->F, J, L.s2, st);
        launch_layer<float, false>(s->dtype, h1, w->wf2, w->bf2, logits, part, B, s->n_answers, s->F, L.s3, st);
    }
    hipLaunchKernelGGL(k_head_softmax, dim3(unsigned((B + 3) / 4)), dim3(256), 0, st, logits, probs, B, s->n_answers);
    HIP_TRY(hipGetLastError(), "dynbatch_classify");
    return DYNB_OK;
}
