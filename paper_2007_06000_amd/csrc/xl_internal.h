// Internal descriptors shared by the host planner and the HIP kernels of libxl.
// Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "xl.h"

namespace xl {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Matrix-core tile geometry.  MF = 32 uses V_MFMA_F32_32X32X2_F32 (one K step of
// the packed filter covers 8 input channels: 2 lane halves x 4 components),
// MF = 16 uses V_MFMA_F32_16X16X4_F32 (16 channels: 4 lane quarters x 4).
// With split-bf16 operands (pr = 1: V_MFMA_F32_32X32X16_BF16 / V_MFMA_F32_16X16X32_BF16, three per
// product) a lane holds 8 channels and a K step covers twice as many.
constexpr int kc_of(int mf, int pr = 0) { return (mf == 32 ? 8 : 16) << pr; }      // channels per K step
constexpr int gps_of(int mf, int pr = 0) { return (mf == 32 ? 2 : 4) << pr; }      // 4-channel groups per K step

// One convolution as the kernels see it.
struct ConvW {
    const f32x4 *wp;        // filter, times the per-channel scale, re-laid out as [K step][tap][row tile][lane] of float4
                            // (split-bf16 kernels: [K step][tap][row tile][hi, lo][lane] of 8 bf16)
    const f32x4 *aff;       // shift in accumulator order: [row tile][quad][lane] float4
    int cin, cout;
    int k, stride, pad;
    int relu;
    int nkg;                // K steps  = ceil(cin / kc)
    int nrt;                // row tiles = ceil(cout / MF)
};

enum Kind { KIND_SINGLE = 0, KIND_FUSED2 = 1, KIND_POOL = 2, KIND_DW = 3, KIND_POOLS = 4, KIND_FUSED2P = 5, KIND_THIN = 6 };

// Kernel argument of every convolution-stage kernel.
//   KIND_SINGLE: stage 1 writes its result to global memory (one layer, the
//                unfused primitive).
//   KIND_FUSED2: stage 1 writes a halo-extended tile of the intermediate into
//                LDS; stage 2 runs one or two sibling convolutions from that
//                tile (straight / split), optionally adding a shortcut tensor
//                in the epilogue (merge).
//   KIND_FUSED2P: KIND_FUSED2 (without shortcut) followed by a max pooling of the block's output: every
//                stage-2 pass leaves its result in an LDS tile, which is pooled before it goes to memory.
//                th x tw is then the stage-2 tile a pth x ptw tile of the pooled output depends on.
//   KIND_POOL:   stage 1 as above; stage 2 is a max pooling from the LDS tile.
//   KIND_POOLS:  KIND_POOL for a first layer whose reduction fits one chunk, as a stream: resident
//                workgroups walk the tiles and request the next tile's input ahead (pool_stream_kernel).
//   KIND_THIN:   a first layer with at most 4 input channels on the vector ALU (thin_conv_kernel): a lane owns
//                a pixel of the tile, filter values are scalar operands; alone (KIND_SINGLE blocks) or followed
//                by a max pooling from an LDS tile (KIND_POOL blocks).
//   KIND_DW:     stage 1 is a depthwise convolution (one filter per channel, vector ALU) into the
//                LDS tile; stage 2 as KIND_FUSED2.  c1.wp / c1.aff then hold the plain depthwise
//                tables ([channel group][tap] and [channel group][scale, shift] float4).
struct BlockParams {
    const float *x;         // block input  [N, Cin, H, W]
    float *y;               // tensor the block writes into [N, Cy, Ho, Wo]
    const float *sc;        // shortcut [N, Csc, Ho, Wo] or nullptr
    int N, Cin, H, W;
    int H1, W1;             // extent of the stage-1 output (the intermediate)
    int Ho, Wo;             // extent of the block output
    int Cy, Csc;
    ConvW c1;
    ConvW c1b;              // second producer of a two-producer merge block (n1 == 2): same geometry as c1
    int n1;                 // stage-1 convolutions whose results are summed in the LDS tile (1 or 2)
    int relu_mid;           // activation applied to that sum
    int coff1;              // channel offset into y when stage 1 writes global
    int n2;                 // stage-2 convolutions (0 for SINGLE / POOL)
    ConvW c2[2];
    int coff2[2];
    int s2;                 // stride shared by the stage-2 windows
    int P2;                 // halo of the LDS tile on the top/left = largest stage-2 pad
    int pool_k;             // KIND_POOL: window size (stride s2, pad P2); KIND_FUSED2P: window size (stride ps2, pad pp)
    int ps2;                // KIND_FUSED2P: stride of the pooling after stage 2
    int pp;                 // KIND_FUSED2P: padding of that pooling (its windows may start above / left of the image)
    int pth, ptw;           // KIND_FUSED2P: tile of the pooled output
    int H2, W2;             // KIND_FUSED2P: extent of the stage-2 output (before pooling)
    int relu_out;           // applied after the shortcut add (merge)
    int gap;                // KIND_SINGLE: the tile is the whole image and y receives the mean over its pixels
    int th, tw;             // output tile of the block
    int mh, mw;             // stage-1 output tile (incl. halo) -- equals th, tw for SINGLE
    int ih, iw;             // input tile (incl. halo)
    int iws;                // pixels per row of the staged input in LDS: iw rounded up to 4
    int tiles_x, tiles_y, csplit;
    int nblocks;            // logical workgroups = N * csplit * tiles_y * tiles_x
    int chunk_kg;           // stage 1: K steps staged per chunk
    int chunk_kg2[2];       // stage 2: K steps of filter staged per chunk, per convolution
    int waves_r1;           // stage-1 waves along the row-tile (Cout) direction
    int waves_r2;           // stage-2 waves along the row-tile direction
    int vw2;                // stage 2 lays output pixels out in virtual rows of vw2 >= tw columns
    unsigned rcp_mw, rcp_vw2, rcp_qrow;   // 2^32 / d + 1 for d = mw, vw2, iws / 4 (0 when d is 1): x / d = mulhi(x, rcp) for x < 65536
    // The same multipliers for the other divisors of the index arithmetic (a division by a run-time value costs
    // about 30 vector instructions, and a vector instruction is paid for in matrix-core time):
    unsigned rcp_tiles, rcp_tcs, rcp_csplit, rcp_tiles_x;   // d = tiles_x * tiles_y, that times csplit, csplit, tiles_x
    unsigned rcp_npo, rcp_pw;       // pooling from an LDS tile: d = pooled pixels per tile, pooled pixels per tile row
    int xs_left;                    // input-tile columns left of the image for the tiles with tx = 0
    unsigned rcp_qpr[2], rcp_upg[2];// input stager: d = 4-pixel units per tile row / per channel group, for tiles that
                                    // start inside the image ([0]) and for the tx = 0 tiles ([1])
    int mid_gstride;        // floats between consecutive 4-channel groups of the LDS tile
    int in_gstride;         // same for the staged input
    int lds_buf_off;        // float offset of the two staging buffers in LDS (after the tile)
    int buf_stride;         // floats per staging buffer
    int w_off1;             // stage 1: float offset of the filter chunk inside a buffer (after the input chunk)
    int stream_wgs;         // KIND_POOLS: resident workgroups wanted; the launch rounds it up to a multiple of 8 and
                            // each workgroup walks tiles L, L + gridDim.x, ...
};

// A compiled kernel variant.
struct Variant {
    int id;
    int kind;
    int mf1, k1, nrt1, npt1;    // stage 1: matrix-core tile, filter size, tiles per wave
    int mf2, nrt2, npt2;        // stage 2: matrix-core tile, tiles per wave (0 when unused)
    int k2a, k2b;               // stage 2 filter sizes, heavier sibling first (0 = absent)
    int sc;                     // 1: adds a shortcut tensor in the epilogue (merge mode)
    int px1;                    // > 0: stage 1 (1x1 filter) reads a planar input chunk, px1 * 64 floats per channel;
                                // < 0: stage 1 uses only -px1 of the 4 channel slots (<= -2 * px1 input channels)
    int pr;                     // 0: fp32 matrix operations; 1: split-bf16 operands (3 bf16 operations per product)
};

// id, kind, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1
#define XL_VARIANT_LIST(X)                                \
    X(0, KIND_SINGLE, 32, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(1, KIND_SINGLE, 32, 1, 2, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(2, KIND_SINGLE, 32, 1, 2, 2, 0, 0, 0, 0, 0, 0, 0)            \
    X(42, KIND_SINGLE, 32, 1, 2, 3, 0, 0, 0, 0, 0, 0, 0)           \
    X(43, KIND_SINGLE, 32, 1, 1, 3, 0, 0, 0, 0, 0, 0, 0)           \
    X(44, KIND_SINGLE, 16, 1, 1, 3, 0, 0, 0, 0, 0, 0, 0)           \
    /* 1x1 first layer with planar input chunks staged by LDS-direct loads (PX1 x 64 floats per channel) */ \
    X(62, KIND_SINGLE, 32, 1, 2, 3, 0, 0, 0, 0, 0, 0, 3)          \
    X(63, KIND_SINGLE, 32, 1, 2, 2, 0, 0, 0, 0, 0, 0, 2)          \
    X(64, KIND_SINGLE, 32, 1, 2, 2, 0, 0, 0, 0, 0, 0, 4)          \
    X(65, KIND_SINGLE, 16, 1, 1, 3, 0, 0, 0, 0, 0, 0, 4)          \
    X(100, KIND_SINGLE, 16, 1, 2, 11, 0, 0, 0, 0, 0, 0, 3)        \
    X(101, KIND_SINGLE, 16, 1, 4, 6, 0, 0, 0, 0, 0, 0, 3)          \
    X(66, KIND_FUSED2, 16, 1, 1, 1, 32, 2, 1, 3, 1, 0, 2)         \
    X(67, KIND_FUSED2, 16, 1, 1, 2, 32, 2, 1, 3, 1, 0, 4)         \
    X(68, KIND_FUSED2, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 4)         \
    X(69, KIND_FUSED2, 16, 1, 3, 2, 32, 2, 1, 3, 1, 0, 2)         \
    X(70, KIND_FUSED2, 16, 1, 3, 2, 32, 2, 1, 3, 1, 0, 4)         \
    X(71, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 1, 0, 4)         \
    X(72, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 3, 1, 0, 4)         \
    X(73, KIND_FUSED2, 32, 1, 1, 1, 16, 1, 2, 3, 1, 0, 2)         \
    X(74, KIND_FUSED2, 16, 1, 1, 1, 32, 1, 1, 5, 0, 0, 4)         \
    X(84, KIND_FUSED2, 16, 1, 1, 2, 32, 1, 1, 5, 0, 0, 4)         \
    X(85, KIND_FUSED2, 16, 1, 1, 2, 16, 1, 2, 5, 0, 0, 4)         \
    X(75, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 1, 0, 0, 2)           \
    /* split blocks with 16-pixel stage-2 tiles, 7 per wave (finer padding of 14-wide tiles) */ \
    X(76, KIND_FUSED2, 16, 1, 1, 2, 16, 1, 7, 3, 1, 0, 4)         \
    X(77, KIND_FUSED2, 16, 1, 1, 3, 16, 1, 7, 3, 1, 0, 4)         \
    X(78, KIND_FUSED2, 32, 1, 1, 1, 16, 1, 7, 3, 1, 0, 4)         \
    X(79, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 7, 3, 1, 0, 2)         \
    X(80, KIND_FUSED2, 16, 1, 3, 2, 16, 1, 7, 3, 1, 0, 4)         \
    X(81, KIND_FUSED2, 16, 1, 3, 2, 16, 1, 7, 3, 1, 0, 2)         \
    X(82, KIND_FUSED2, 32, 1, 2, 1, 16, 1, 7, 3, 1, 0, 4)         \
    X(83, KIND_FUSED2, 16, 1, 1, 2, 16, 1, 7, 3, 1, 0, 0)           \
    X(3, KIND_SINGLE, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(4, KIND_SINGLE, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(5, KIND_SINGLE, 32, 3, 2, 2, 0, 0, 0, 0, 0, 0, 0)            \
    X(6, KIND_SINGLE, 16, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(7, KIND_SINGLE, 16, 1, 1, 2, 0, 0, 0, 0, 0, 0, 0)            \
    X(8, KIND_SINGLE, 16, 1, 3, 2, 0, 0, 0, 0, 0, 0, 0)            \
    X(9, KIND_SINGLE, 16, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(10, KIND_SINGLE, 16, 3, 1, 2, 0, 0, 0, 0, 0, 0, 0)           \
    /* 3x3 layers on small images: 16-pixel tiles, three per wave (13x13 = 169 pixels pad to 176, in 12 slots) */ \
    X(150, KIND_SINGLE, 16, 3, 1, 3, 0, 0, 0, 0, 0, 0, 0)          \
    X(151, KIND_SINGLE, 16, 3, 2, 3, 0, 0, 0, 0, 0, 0, 0)          \
    X(152, KIND_SINGLE, 16, 3, 2, 2, 0, 0, 0, 0, 0, 0, 0)          \
    /* split (fire-like): 1x1 -> {3x3, 1x1} */            \
    X(11, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 1, 0, 0)          \
    X(12, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 3, 1, 0, 0)          \
    X(13, KIND_FUSED2, 16, 1, 1, 1, 32, 2, 1, 3, 1, 0, 0)          \
    X(14, KIND_FUSED2, 16, 1, 1, 2, 32, 2, 1, 3, 1, 0, 0)          \
    X(15, KIND_FUSED2, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 0)          \
    X(16, KIND_FUSED2, 16, 1, 3, 2, 32, 2, 1, 3, 1, 0, 0)          \
    X(17, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 3, 1, 0, 0)          \
    X(18, KIND_FUSED2, 32, 1, 1, 1, 16, 1, 2, 3, 1, 0, 0)          \
    /* split -> max pooling of the concatenated result */  \
    X(110, KIND_FUSED2P, 32, 1, 1, 1, 32, 2, 1, 3, 1, 0, 0)        \
    X(111, KIND_FUSED2P, 32, 1, 2, 1, 32, 2, 1, 3, 1, 0, 0)        \
    X(112, KIND_FUSED2P, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 0)        \
    X(113, KIND_FUSED2P, 16, 1, 3, 2, 32, 2, 1, 3, 1, 0, 0)        \
    X(114, KIND_FUSED2P, 32, 1, 1, 1, 16, 1, 2, 3, 1, 0, 0)        \
    X(115, KIND_FUSED2P, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 4)        \
    X(116, KIND_FUSED2P, 16, 1, 1, 3, 16, 1, 7, 3, 1, 0, 4)        \
    X(117, KIND_FUSED2P, 16, 1, 1, 2, 32, 2, 1, 3, 1, 0, 0)        \
    X(118, KIND_FUSED2P, 16, 1, 2, 3, 32, 2, 1, 3, 1, 0, 0)        \
    X(119, KIND_FUSED2P, 32, 1, 1, 2, 32, 2, 1, 3, 1, 0, 0)        \
    X(120, KIND_FUSED2P, 16, 1, 1, 4, 32, 2, 1, 3, 1, 0, 0)        \
    /* straight conv -> conv, and merge (with shortcut) */ \
    X(19, KIND_FUSED2, 32, 3, 2, 1, 32, 2, 1, 3, 0, 0, 0)          \
    X(20, KIND_FUSED2, 32, 3, 2, 1, 32, 2, 1, 3, 0, 1, 0)          \
    X(21, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 3, 0, 0, 0)          \
    X(22, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 3, 0, 1, 0)          \
    X(23, KIND_FUSED2, 16, 3, 1, 1, 16, 1, 2, 3, 0, 0, 0)          \
    X(24, KIND_FUSED2, 16, 3, 1, 3, 16, 1, 2, 3, 0, 0, 0)          \
    X(25, KIND_FUSED2, 16, 3, 1, 1, 16, 1, 2, 3, 0, 1, 0)          \
    X(26, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 0, 0, 0)          \
    X(27, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 1, 0, 0, 0)          \
    X(28, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 1, 0, 0, 0)          \
    X(29, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 1, 0, 0, 0)          \
    X(30, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 3, 0, 0, 0)          \
    X(31, KIND_FUSED2, 16, 3, 1, 1, 16, 1, 2, 1, 0, 0, 0)          \
    X(60, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 1, 0, 0, 0)          \
    X(61, KIND_FUSED2, 16, 1, 2, 2, 16, 1, 2, 1, 0, 0, 0)          \
    X(32, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 1, 0, 1, 0)          \
    X(33, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 0, 1, 0)          \
    X(34, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 1, 0, 1, 0)          \
    X(35, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 3, 0, 1, 0)          \
    /* stage 2 on 16-pixel tiles, 7 per wave: finer padding of small tiles */ \
    X(45, KIND_FUSED2, 32, 3, 2, 1, 16, 1, 7, 3, 0, 1, 0)          \
    X(46, KIND_FUSED2, 32, 3, 2, 1, 16, 1, 7, 3, 0, 0, 0)          \
    /* 5x5 filters (paper Table 1, a.1: 1x1 -> 5x5) and their unfused forms */ \
    X(47, KIND_SINGLE, 32, 5, 1, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(48, KIND_SINGLE, 32, 5, 2, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(49, KIND_SINGLE, 16, 5, 1, 2, 0, 0, 0, 0, 0, 0, 0)             \
    X(50, KIND_FUSED2, 16, 1, 1, 1, 32, 1, 1, 5, 0, 0, 0)            \
    X(51, KIND_FUSED2, 16, 1, 1, 2, 32, 1, 1, 5, 0, 0, 0)            \
    X(52, KIND_FUSED2, 32, 1, 1, 1, 32, 1, 1, 5, 0, 0, 0)            \
    X(53, KIND_FUSED2, 16, 1, 1, 1, 16, 1, 2, 5, 0, 0, 0)            \
    X(54, KIND_FUSED2, 32, 3, 1, 1, 32, 1, 1, 5, 0, 0, 0)            \
    /* depthwise -> pointwise (paper Table 1, a.2); MF1 / NRT1 / NPT1 unused */ \
    X(55, KIND_DW, 32, 3, 1, 1, 32, 2, 1, 1, 0, 0, 0)                \
    X(56, KIND_DW, 32, 3, 1, 1, 32, 1, 1, 1, 0, 0, 0)                \
    X(57, KIND_DW, 32, 3, 1, 1, 16, 1, 2, 1, 0, 0, 0)                \
    X(58, KIND_DW, 32, 3, 1, 1, 32, 2, 1, 3, 0, 0, 0)                \
    X(59, KIND_DW, 32, 3, 1, 1, 16, 1, 2, 3, 0, 0, 0)                \
    /* conv -> maxpool as a stream of tiles (first layer of one chunk) */ \
    X(94, KIND_POOLS, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(95, KIND_POOLS, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(96, KIND_POOLS, 16, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(97, KIND_POOLS, 32, 1, 2, 1, 0, 0, 0, 0, 0, 0, 0)           \
    /* ... with at most 4 input channels packed two per channel slot (PX1 = -2: 2 of 4 slots used) */ \
    X(98, KIND_POOLS, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, -2)          \
    X(99, KIND_POOLS, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, -2)          \
    /* thin first layers (at most 4 input channels) on the vector ALU, alone or with a max pooling from an LDS tile: \
       columns are id, kind, -, K, Cin, -, -, -, -, -, pooling window (0: none), then unused */ \
    X(130, KIND_THIN, 32, 3, 3, 1, 0, 0, 0, 0, 3, 0, 0)           \
    X(131, KIND_THIN, 32, 3, 3, 1, 0, 0, 0, 0, 2, 0, 0)           \
    X(132, KIND_THIN, 32, 3, 3, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(133, KIND_THIN, 32, 3, 4, 1, 0, 0, 0, 0, 3, 0, 0)           \
    X(134, KIND_THIN, 32, 3, 4, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(135, KIND_THIN, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(136, KIND_THIN, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(137, KIND_THIN, 32, 5, 3, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(138, KIND_THIN, 32, 1, 3, 1, 0, 0, 0, 0, 0, 0, 0)           \
    X(139, KIND_THIN, 32, 1, 4, 1, 0, 0, 0, 0, 0, 0, 0)           \
    /* ... 3x3 stride 2 -> pooling 3x3 stride 2 with a 2x2 block of convolution outputs per lane (column 6 = 2) */ \
    X(140, KIND_THIN, 32, 3, 3, 2, 0, 0, 0, 0, 3, 0, 0)           \
    X(141, KIND_THIN, 32, 3, 1, 2, 0, 0, 0, 0, 3, 0, 0)           \
    /* conv -> maxpool */                                 \
    X(36, KIND_POOL, 32, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(37, KIND_POOL, 32, 1, 2, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(38, KIND_POOL, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(39, KIND_POOL, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(40, KIND_POOL, 16, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)             \
    X(41, KIND_POOL, 16, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)

// Variants with split-bf16 operands (ids from 200): same columns.  Stage 2 uses 32-row tiles only, so
// that its K step (16 channels) divides what stage 1 writes into the LDS tile (whole 16- or 32-row tiles).
#define XL_VARIANT_LIST_B3(X)                                      \
    X(200, KIND_SINGLE, 32, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(201, KIND_SINGLE, 32, 1, 2, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(202, KIND_SINGLE, 32, 1, 2, 2, 0, 0, 0, 0, 0, 0, 0)          \
    X(204, KIND_SINGLE, 16, 1, 1, 3, 0, 0, 0, 0, 0, 0, 0)          \
    X(205, KIND_SINGLE, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(206, KIND_SINGLE, 32, 3, 2, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(207, KIND_SINGLE, 32, 3, 2, 2, 0, 0, 0, 0, 0, 0, 0)          \
    X(208, KIND_SINGLE, 32, 5, 1, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(209, KIND_SINGLE, 32, 1, 2, 3, 0, 0, 0, 0, 0, 0, 0)          \
    X(214, KIND_SINGLE, 32, 1, 4, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(216, KIND_SINGLE, 32, 3, 4, 1, 0, 0, 0, 0, 0, 0, 0)          \
    X(217, KIND_SINGLE, 32, 3, 1, 2, 0, 0, 0, 0, 0, 0, 0)          \
    X(218, KIND_SINGLE, 16, 3, 1, 2, 0, 0, 0, 0, 0, 0, 0)          \
    X(203, KIND_SINGLE, 32, 1, 2, 4, 0, 0, 0, 0, 0, 0, 0)          \
    X(222, KIND_FUSED2, 32, 3, 2, 2, 32, 2, 2, 3, 0, 0, 0)         \
    X(213, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 2, 3, 1, 0, 0)         \
    /* split */                                                    \
    X(210, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 1, 0, 0)         \
    X(211, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 3, 1, 0, 0)         \
    X(212, KIND_FUSED2, 16, 1, 1, 2, 32, 2, 1, 3, 1, 0, 0)         \
    X(233, KIND_FUSED2, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 0)         \
    X(235, KIND_FUSED2, 16, 1, 3, 2, 32, 2, 1, 3, 1, 0, 0)         \
    /* split -> max pooling */                                     \
    X(250, KIND_FUSED2P, 32, 1, 1, 1, 32, 2, 1, 3, 1, 0, 0)        \
    X(251, KIND_FUSED2P, 16, 1, 1, 3, 32, 2, 1, 3, 1, 0, 0)        \
    X(252, KIND_FUSED2P, 16, 1, 2, 3, 32, 2, 1, 3, 1, 0, 0)        \
    X(253, KIND_FUSED2P, 32, 1, 1, 2, 32, 2, 1, 3, 1, 0, 0)        \
    /* straight and merge */                                       \
    X(220, KIND_FUSED2, 32, 3, 2, 1, 32, 2, 1, 3, 0, 0, 0)         \
    X(221, KIND_FUSED2, 32, 3, 2, 1, 32, 2, 1, 3, 0, 1, 0)         \
    X(224, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 3, 0, 0, 0)         \
    X(225, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 3, 0, 1, 0)         \
    X(226, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 0, 0, 0)         \
    X(227, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 3, 0, 1, 0)         \
    X(228, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 1, 0, 0, 0)         \
    X(229, KIND_FUSED2, 32, 1, 1, 1, 32, 2, 1, 1, 0, 1, 0)         \
    X(230, KIND_FUSED2, 32, 3, 1, 1, 32, 2, 1, 1, 0, 0, 0)         \
    X(231, KIND_FUSED2, 16, 1, 1, 1, 32, 1, 1, 5, 0, 0, 0)         \
    /* two producers -> add -> consumer, all 1x1 */                \
    X(254, KIND_FUSED2, 32, 1, 2, 1, 32, 2, 1, 1, 0, 0, 0)         \
    /* depthwise (vector ALU, fp32) -> convolution on split-bf16 operands */ \
    X(255, KIND_DW, 32, 3, 1, 1, 32, 2, 1, 1, 0, 0, 0)             \
    X(256, KIND_DW, 32, 3, 1, 1, 32, 1, 1, 1, 0, 0, 0)             \
    X(257, KIND_DW, 32, 3, 1, 1, 32, 2, 1, 3, 0, 0, 0)             \
    /* conv -> maxpool (the LDS tile stays fp32) */                \
    X(240, KIND_POOL, 32, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0)            \
    X(241, KIND_POOL, 32, 3, 1, 1, 0, 0, 0, 0, 0, 0, 0)

const std::vector<Variant> &variants();

#ifndef XL_STAGE_UNITS
#define XL_STAGE_UNITS 1
#endif
constexpr int STAGE_UNITS = XL_STAGE_UNITS;      // input units (4 channels x 4 pixels) each thread stages per chunk
constexpr int MAX_W_CHUNK_BYTES = 52 * 1024;  // filter bytes staged per chunk (LDS-direct loads, no registers)
constexpr int PLANAR_SLOTS = 8;     // LDS-direct loads per wave and chunk of a planar input chunk
constexpr int MAX_THREADS = 512;
// floats per filter row of the thin layout: the taps rounded up to whole 64-byte lines, so that a row is read by
// aligned 64-byte scalar loads (the scalar cache serves requests, not bytes: a row that straddles lines costs more)
constexpr int thin_row_floats(int taps) { return (taps + 15) / 16 * 16; }
constexpr int THIN_PCB = 4;         // thin_conv_pool_kernel: output channels per LDS tile (per barrier)
constexpr int MAX_ALTERNATIVES = 64;  // candidates per block kept for on-device tuning
#ifndef XL_MIN_WAVES
#define XL_MIN_WAVES 2
#endif

// ---- launchers (kernels.hip) -------------------------------------------------
hipError_t launch_block(int variant, const BlockParams &p, int threads, size_t lds_bytes, hipStream_t s);
hipError_t configure_kernels(int max_lds_bytes);      // raises the dynamic-LDS cap of every variant

hipError_t launch_pack_filter(const float *w, const float *scale, f32x4 *wp, int cout, int cin, int k, int mf,
                              int nkg, int nrt, hipStream_t s, int pairs = 0, int pr = 0);
// peak probes: 0 = copy (bytes from src to dst), 1 = fp32 matrix loop, 2 = bf16 matrix loop, 3 = fp32 multiply-add loop;
// `work` receives bytes moved or floating-point operations issued by one launch
hipError_t launch_peak_probe(int what, void *dst, const void *src, size_t bytes, int num_cus, hipStream_t s, double *work);
hipError_t launch_pack_thin(const float *w, const float *scale, const float *shift, float *wp, float *aff, int cout,
                            int taps, hipStream_t s);
hipError_t launch_pack_affine(const float *shift, f32x4 *out, int cout, int mf, int nrt, hipStream_t s);
hipError_t launch_maxpool(const float *x, float *y, int N, int C, int H, int W, int Ho, int Wo,
                          int k, int stride, int pad, int Cy, int coff, hipStream_t s);
hipError_t launch_add(const float *a, const float *b, float *y, long long count, int relu, hipStream_t s);
hipError_t launch_gap(const float *x, float *y, int NC, int HW, hipStream_t s);
hipError_t launch_pack_depthwise(const float *w, const float *scale, const float *shift, f32x4 *wp, f32x4 *aff, int C,
                                 int k, hipStream_t s);
hipError_t launch_depthwise(const float *x, float *y, const f32x4 *wp, const f32x4 *aff, int N, int C, int H, int W,
                            int Ho, int Wo, int k, int stride, int pad, int relu, int Cy, int coff, hipStream_t s);

}  // namespace xl
