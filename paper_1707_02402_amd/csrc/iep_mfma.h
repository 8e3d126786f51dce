// MFMA building blocks of the fused module kernels (bf16, C = 128, 14 x 14), shared by the forward executor and the
// backward pass: the LDS halo tile's geometry, the packed weight fragment order and the software-pipelined K loop.
#pragma once

#include <hip/hip_runtime.h>

#include "device_utils.h"

namespace {

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
constexpr int CENTER = ROW_BYTES + PIX_BYTES;           // (+1,+1) from the top-left tap
}  // namespace mf

__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t addr)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    return *reinterpret_cast<const bf16x8*>(lds_raw + addr);
}

// ---- MFMA tiling ------------------------------------------------------------------------------
// v_mfma_f32_32x32x16_bf16 is the efficient bf16 instruction of gfx950 (measured: ~2.1 PFLOP/s chip
// wide, against ~1.5 for the 16x16x32 form), so a convolution is tiled as
//     D[32 channels][32 pixels] += W[32 channels][16 k] * X[16 k][32 pixels]
// with the weights as the A operand and the activations as the B operand: a lane then ends up with
// 16 channels of one pixel (consecutive ones, thanks to the row permutation of the packed weights),
// which it can store as 16-byte pieces.  196 pixels make 7 pixel tiles (224 rows, the last 28 are
// padding).  A wave owns one channel tile and all pixel tiles of its node.
//
// K order.  Within a tap the 128 input channels are consumed in 8 steps of 16; lane half h = lane/32
// supplies channels h*64 + j*8 .. +7 in step j (any pairing works as long as both operands agree).
// Weight fragments.  In the caller's [Cout][kh][kw][Cin] layout one fragment load would touch 64
// different cache lines (32 rows x 2 halves), which makes the vector L1 the bottleneck.  The
// weights are therefore repacked (k_pack_weights) into fragment order
//     [function][channel tile 4][tap][step 8][lane 64][8 bf16]
// so that the 64 lanes of a fragment load read one contiguous kilobyte.
constexpr int MT7 = 7;

namespace mf {
constexpr int FRAG = 512;   // elements of one packed weight fragment: 64 lanes x 8 bf16 = 1 KB
}

// ---- K loop -----------------------------------------------------------------------------------------
// acc[t][nt] += W * X over one 3x3 convolution (9 taps x 8 steps of 16 input channels) or, CENTER_ONLY, over the
// 8 steps of the centre tap (one half of the 1x1 convolution).  Software pipelined by hand:
//   * activation fragments live in XS register sets; the LDS reads that fill the set of the step XS/2 ahead are
//     interleaved one by one with the MFMAs of the current step, so LDS traffic is spread evenly under them;
//   * weight fragments live in a ring of RW steps (the caller's registers); the slot of the previous step is
//     refilled from global memory right after the first pixel tile of the current step, RW - 1 steps ahead of its
//     use (issuing the load directly behind the MFMAs that still read the slot would stall the wave);
//   * scheduler fences keep that order (the compiler would otherwise sink every load to its use).
// The ring is filled by ring_fill, a call of its own so that the caller can issue it long before the loop; the
// last chunk refills the ring with the first fragments of the NEXT loop (wnext), which then starts full.
// Measured on this chip: a workgroup receives about 27 bytes per clock of weight fragments whatever the
// look-ahead, so a loop is only MFMA-bound if every fragment is fetched once per workgroup: each wave owns one
// channel tile (32 output channels) and all pixel tiles of its node (NT = 1); with two nodes per workgroup a
// wave would own NT = 2 channel tiles of one node.
template <int NT, int RW>
__device__ __forceinline__ void ring_fill(bf16x8 (&wf)[RW][NT], const bf16_t* (&wrow)[NT])
{
#pragma unroll
    for (int j = 0; j < RW - 1; ++j) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wf[j][nt] = *reinterpret_cast<const bf16x8*>(wrow[nt] + j * mf::FRAG);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int MTW, int NT, int RW, int XS, bool CENTER_ONLY>
__device__ __forceinline__ void kloop(f32x16 (&acc)[MTW][NT], const uint32_t (&xaddr)[MTW], bf16x8 (&wf)[RW][NT],
                                      const bf16_t* (&wrow)[NT], const bf16_t* (&wnext)[NT])
{
    constexpr int NSTEP = CENTER_ONLY ? 8 : 72;
    constexpr int NCHUNK = NSTEP / RW, XA = XS / 2;
    static_assert(NSTEP % RW == 0 && RW % 8 == 0 && RW % XS == 0 && (XS == 2 || XS == 4), "ring shapes");
    static_assert(RW == 8 || RW == 24, "a chunk is one tap or one kernel row");
    // byte offset of step j (0 .. RW) of a chunk from the chunk's first tap: taps advance by a pixel, steps by 16 bytes
    auto in_chunk = [](int j) -> uint32_t { return uint32_t((j / 8) * mf::PIX_BYTES + (j % 8) * 16); };
    auto chunk_base = [](int c) -> uint32_t {
        if (CENTER_ONLY) return uint32_t(mf::CENTER);
        if (RW == 24) return uint32_t(c) * mf::ROW_BYTES;
        return uint32_t(c / 3) * mf::ROW_BYTES + uint32_t(c % 3) * mf::PIX_BYTES;
    };
    bf16x8 x[XS][MTW];
#pragma unroll
    for (int jj = 0; jj < XA; ++jj)
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            x[jj][t] = lds_read_frag(xaddr[t] + chunk_base(0) + in_chunk(jj));
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll 1
    for (int c = 0; c < NCHUNK; ++c) {
        const bool last = c + 1 >= NCHUNK;
        uint32_t xa[MTW], xn[MTW];                      // this chunk's and the next chunk's activations
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            xa[t] = xaddr[t] + chunk_base(c);
            xn[t] = xaddr[t] + chunk_base(last ? c : c + 1);        // after the last chunk: re-read valid data
        }
        const bf16_t* cur[NT];                          // fragment RW - 1 of this chunk
        const bf16_t* nxt[NT];                          // fragments 0 .. RW - 2 of the next chunk / the next loop
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            cur[nt] = wrow[nt] + (c * RW + RW - 1) * mf::FRAG;
            nxt[nt] = last ? wnext[nt] : wrow[nt] + (c + 1) * RW * mf::FRAG;
        }
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            const int ja = j + XA;                      // the step whose activations are fetched now
#pragma unroll
            for (int t = 0; t < MTW; ++t) {
                x[ja % XS][t] = lds_read_frag(ja >= RW ? xn[t] + in_chunk(ja - RW) : xa[t] + in_chunk(ja));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[t][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][nt], x[j % XS][t], acc[t][nt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (t == 0) {                           // refill the slot of the previous step
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        wf[(j + RW - 1) % RW][nt] = j == 0 ? *reinterpret_cast<const bf16x8*>(cur[nt])
                                                           : *reinterpret_cast<const bf16x8*>(nxt[nt] + (j - 1) * mf::FRAG);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
}

}  // namespace
