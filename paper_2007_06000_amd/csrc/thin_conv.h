// Thin first layers on the vector ALU (included by kernels.hip).
//
// A convolution with a handful of input channels (the 3-channel stem of an image network) gives the
// matrix cores a reduction of 27 terms: most of a K step is padding, and the layer is bound by moving
// its input and output, not by arithmetic (paper section 2.2: convolutions with few input channels are
// memory-bound).  Here it runs as plain multiply-adds instead:
//   - a lane owns one PIXEL of the workgroup's tile of convolution outputs and keeps that pixel's whole
//     input window, Cin * K * K values, in registers (loaded once, every load in flight together);
//   - the output channels are looped over; a filter value is the same for every lane, so it is not
//     vector data at all: the filter is read with scalar loads (wave-uniform addresses, constant
//     address space; it is a few KB and stays in the scalar cache) and enters v_fmac_f32 as its scalar
//     operand.  No filter in LDS, no staging through registers;
//   - a following max pooling (paper Fig. 3b: Layer2 consumes Layer1's output on chip) takes the
//     convolution outputs of 8 channels at a time from an LDS tile (two tiles alternate, one barrier
//     per 8 channels): the convolution output never reaches HBM.  Bias and ReLU are applied after the
//     maximum (both are monotonic, so the result is bit-identical to applying them first).  PK is the
//     pooling window (0: no pooling); which pooled pixels a lane takes does not depend on the channel
//     chunk and is worked out once.
//   - without a pooling the lanes store their outputs directly (consecutive lanes = consecutive pixels
//     of a tile row).
// thin_conv_pool_kernel below is the faster form for the one shape that matters most (3x3 stride 2 -> pooling 3x3
// stride 2); this one covers every other filter size, stride and pooling.
//
// BlockParams fields used: x, y, N, Cin, H, W, H1, W1 (convolution output extent), Ho, Wo (block output
// extent), Cy, coff1, c1 (wp: filter as [Cout rounded up to 16][Cin*K*K rounded up to 16] floats with the scale folded
// in, aff: shift as [Cout rounded up to 16] floats; stride, pad, relu, cout), pool_k (0: no pooling),
// s2 / P2 (stride / padding of the pooling), th x tw (output tile), mh x mw (tile of convolution outputs
// under it, at most blockDim.x pixels), rcp_mw, rcp_vw2 (for tw), rcp_qrow (for th * tw), tiles_x,
// tiles_y, nblocks.  LDS: two tiles of THIN_OCB x blockDim.x floats.
#pragma once

namespace xl {

constexpr int THIN_OCB = 8;         // output channels per LDS tile (per barrier)

template <int CIN, int K, int PK>
__global__ void __launch_bounds__(MAX_THREADS) thin_conv_kernel(const BlockParams P)
{
    constexpr int T = CIN * K * K;
    constexpr int RS = thin_row_floats(T);      // filter rows start on 64-byte lines: a row is whole 64-byte scalar loads
    constexpr int OCB = THIN_OCB;
    typedef const float __attribute__((address_space(4))) cfloat;    // read-only, wave-uniform: scalar loads
    extern __shared__ __attribute__((aligned(16))) float lds[];

    const int L = logical_block();
    if (L >= P.nblocks) return;
    const int tiles = P.tiles_x * P.tiles_y;
    const int tile = L % tiles, n = L / tiles;
    const int ty = tile / P.tiles_x, tx = tile - ty * P.tiles_x;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const bool pooled = P.pool_k > 0;
    const int oy0 = ty * P.th, ox0 = tx * P.tw;                         // first output pixel of the tile
    const int my0 = pooled ? oy0 * P.s2 - P.P2 : oy0;                   // first convolution output under it
    const int mx0 = pooled ? ox0 * P.s2 - P.P2 : ox0;
    const int npx = P.mh * P.mw;

    // ---- this lane's pixel and its input window
    const int r = fdiv(tid, P.rcp_mw), c = tid - r * P.mw;
    const int cy = my0 + r, cx = mx0 + c;
    const bool valid = tid < npx && cy >= 0 && cy < P.H1 && cx >= 0 && cx < P.W1;
    const int H = P.H, W = P.W, S = P.c1.stride, pad = P.c1.pad;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(P.x + (size_t)n * CIN * H * W,
                                                (unsigned long long)(P.N - n) * CIN * H * W * 4ull);
    float x[T];
    {
        const int gy0 = cy * S - pad, gx0 = cx * S - pad;
#pragma unroll
        for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
            for (int u = 0; u < K; ++u)
#pragma unroll
                for (int v = 0; v < K; ++v) {
                    const int gy = gy0 + u, gx = gx0 + v;
                    const bool in = valid && gy >= 0 && gy < H && gx >= 0 && gx < W;
                    // a lane without an element aims past the end of the buffer: the load returns zero
                    const unsigned off = in ? (unsigned)(((ci * H + gy) * W + gx) * 4) : 0xfffffff0u;
                    x[(ci * K + u) * K + v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xr, off, 0, 0));
                }
    }

    const int cout = P.c1.cout;
    const int nchunks = (cout + OCB - 1) / OCB;
    cfloat *wq = (cfloat *)(unsigned long long)P.c1.wp;
    cfloat *shift_s = (cfloat *)(unsigned long long)P.c1.aff;                  // by scalar loads (uniform channel)
    const size_t oplane = (size_t)P.Ho * P.Wo;
    const __amdgpu_buffer_rsrc_t yr = make_rsrc(P.y + ((size_t)n * P.Cy + P.coff1) * oplane,
                                                ((unsigned long long)(P.N - n) * P.Cy - P.coff1) * oplane * 4ull);

    if constexpr (PK == 0) {
        const unsigned own = (unsigned)((cy * P.Wo + cx) * 4);                // this lane's output pixel
        for (int oc = 0; oc < cout; ++oc) {
            cfloat *wr = wq + (size_t)oc * RS;
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < T; ++t) acc = fmaf(x[t], wr[t], acc);
            float z = acc + shift_s[oc];
            if (P.c1.relu) z = fmaxf(z, 0.f);
            if (valid) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, z), yr, own, oc * (int)oplane * 4, 0);
        }
    } else {
        // ---- the pooled pixels this lane takes in every chunk: item = (channel of the chunk, pooled pixel), pixels
        // of a row on consecutive lanes.  NI items cover workgroups of stride-2 poolings; the rare rest is
        // worked out on the fly.
        constexpr int NI = 4;
        const int ntile = P.th * P.tw;
        const int nitems = OCB * ntile;
        const float *shift_v = reinterpret_cast<const float *>(P.c1.aff);     // the shifts, for lanes that differ in channel
        int i_src[NI], i_o[NI];
        unsigned i_dst[NI];
        auto item = [&](int it, int &src, int &o, unsigned &dst) {
            o = fdiv(it, P.rcp_qrow);
            const int q = it - o * ntile;
            const int py = fdiv(q, P.rcp_vw2), px = q - py * P.tw;
            const int gy = oy0 + py, gx = ox0 + px;
            src = o * nthreads + (py * P.s2) * P.mw + px * P.s2;
            dst = (gy < P.Ho && gx < P.Wo) ? (unsigned)((gy * P.Wo + gx) * 4) : ~0u;      // ~0: nothing to store
        };
#pragma unroll
        for (int k = 0; k < NI; ++k) item(min(tid + k * nthreads, nitems - 1), i_src[k], i_o[k], i_dst[k]);
#pragma unroll
        for (int k = 0; k < NI; ++k)
            if (tid + k * nthreads >= nitems) i_dst[k] = ~0u;
        auto pool_store = [&](const float *buf, int ch, int src, int o, unsigned dst, float sh) {
            const int oc = ch * OCB + o;
            const float *sp = buf + src;
            float m = sp[0];
#pragma unroll
            for (int u = 0; u < PK; ++u)
#pragma unroll
                for (int v = 0; v < PK; ++v)
                    if (u + v > 0) m = fmaxf(m, sp[u * P.mw + v]);
            m += sh;
            if (P.c1.relu) m = fmaxf(m, 0.f);
            // (the channel differs from lane to lane here: it goes into the lane's own offset, not the scalar one)
            if (oc < cout && dst != ~0u)
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, m), yr, dst + (unsigned)(oc * (int)oplane * 4), 0, 0);
        };
        for (int ch = 0; ch < nchunks; ++ch) {
            float *buf = lds + (ch & 1) * OCB * nthreads;
            // the shifts of this lane's pooled items: requested now, needed after the multiply-adds
            float sh[NI];
#pragma unroll
            for (int k = 0; k < NI; ++k) sh[k] = shift_v[ch * OCB + i_o[k]];
            // two channels at a time: their filter rows arrive with one wait, and the two chains of multiply-adds
            // alternate
            for (int o = 0; o < OCB; o += 2) {
                cfloat *wr = wq + (size_t)(ch * OCB + o) * RS;
                float w0[T], w1[T];
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    w0[t] = wr[t];
                    w1[t] = wr[RS + t];
                }
                float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    acc0 = fmaf(x[t], w0[t], acc0);
                    acc1 = fmaf(x[t], w1[t], acc1);
                }
                // outside the layer's extent the pooling must not look (section 3.3: the tile is written with the
                // next layer's padding value already in place)
                buf[o * nthreads + tid] = valid ? acc0 : -FLT_MAX;
                buf[(o + 1) * nthreads + tid] = valid ? acc1 : -FLT_MAX;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < NI; ++k)
                if (k * nthreads < nitems) pool_store(buf, ch, i_src[k], i_o[k], i_dst[k], sh[k]);
            for (int it = tid + NI * nthreads; it < nitems; it += nthreads) {
                int src, o;
                unsigned dst;
                item(it, src, o, dst);
                pool_store(buf, ch, src, o, dst, shift_v[ch * OCB + o]);
            }
            // the next chunk goes to the other tile; this one is overwritten two chunks on, after the barrier in between
        }
    }
}

// ----------------------------------------------------------------------------
// The stem of an image network in one shape: convolution 3x3 with stride 2 followed by max pooling 3x3 with
// stride 2 and no padding (paper Fig. 3b with the layer pair of section 4.2's first block).
//
// Both thin kernels are bound by the vector ALU, and a multiply-add whose filter value is a scalar operand issues
// every 4 cycles per wavefront where one with vector operands only issues every 2.8 (measured: 76 against 110
// TFLOP/s over the chip); every way of putting a wave-uniform value into a vector register instead (an LDS or
// memory read with one address for all lanes, a move) costs more than that difference.  What is left is the
// work around the multiply-adds, and this kernel has less of it: a lane owns the 2x2 block of convolution
// outputs under one pooled pixel, whose 5x5 input window per channel (75 values for 3 channels, loaded as one
// 16-byte and one 4-byte piece per row) it keeps in registers, so a filter value feeds four multiply-adds.
// The pooling window of pooled pixel (py, px) is the lane's own block plus the left column of the block to its
// right, the top row of the block below and the top-left value of the diagonal one, so a lane reduces its block
// to four maxima (all, left column, top row, top-left), passes three of them through LDS, and pools, adds the
// shift, activates and stores its OWN pooled pixel: no remapping of lanes between the two layers, three LDS
// reads per result instead of nine.  Four channels per barrier, two LDS tiles alternate.
//
// BlockParams fields used: x, y, N, H, W, H1, W1, Ho, Wo, Cy, coff1, c1 (wp / aff as thin_conv_kernel, pad, relu,
// cout), th x tw (pooled tile), mw = tw + 1 with rcp_mw, tiles_x, tiles_y, rcp_tiles, rcp_tiles_x, nblocks.
// Lanes: (th + 1) x (tw + 1) blocks, row-major; the last row and column only supply neighbours.
// LDS: 2 tiles of THIN_PCB channels x 3 values x blockDim.x floats.
template <int CIN>
__global__ void __launch_bounds__(256) thin_conv_pool_kernel(const BlockParams P)
{
    constexpr int T = CIN * 9, CB = THIN_PCB;
    constexpr int RS = thin_row_floats(T);
    typedef const float __attribute__((address_space(4))) cfloat;
    typedef unsigned u32x4 __attribute__((vector_size(16)));
    extern __shared__ __attribute__((aligned(16))) float lds[];

    const int L = logical_block();
    if (L >= P.nblocks) return;
    const int tiles = P.tiles_x * P.tiles_y;
    const int n = udiv(L, tiles, P.rcp_tiles), tile = L - n * tiles;
    const int ty = udiv(tile, P.tiles_x, P.rcp_tiles_x), tx = tile - ty * P.tiles_x;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int bw = P.tw + 1;
    const int by = fdiv(tid, P.rcp_mw), bx = tid - by * bw;
    const bool lane_on = tid < (P.th + 1) * bw;
    const int py = ty * P.th + by, px = tx * P.tw + bx;         // this lane's pooled pixel (or a neighbour-only block)
    const int cy0 = 2 * py, cx0 = 2 * px;                       // first convolution output of the block
    const int H = P.H, W = P.W, pad = P.c1.pad;
    const int gy0 = 2 * cy0 - pad, gx0 = 2 * cx0 - pad;         // first input row / column of the block's window

    // ---- the window: 5 rows x 5 columns per input channel
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(P.x + (size_t)n * CIN * H * W, (unsigned long long)(P.N - n) * CIN * H * W * 4ull);
    float x[CIN][5][5];
    if (pad == 0) {
        // Rows below the image and blocks right of it aim past the end of the buffer (zeros).  A piece that
        // starts inside a row may run over its end into the next row: those values only reach convolution
        // outputs at or beyond W1, which are discarded below.
#pragma unroll
        for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
            for (int r = 0; r < 5; ++r) {
                const int gy = gy0 + r;
                const bool in = lane_on && gy < H && gx0 < W;
                const unsigned off = in ? (unsigned)(((ci * H + gy) * W + gx0) * 4) : 0xfffffff0u;
                const f32x4 q = __builtin_bit_cast(f32x4, (u32x4)__builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0));
                const unsigned e = __builtin_amdgcn_raw_buffer_load_b32(xr, in ? off + 16u : 0xfffffff0u, 0, 0);
                x[ci][r][0] = q.x;
                x[ci][r][1] = q.y;
                x[ci][r][2] = q.z;
                x[ci][r][3] = q.w;
                x[ci][r][4] = __builtin_bit_cast(float, e);
            }
    } else {
#pragma unroll
        for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
            for (int r = 0; r < 5; ++r)
#pragma unroll
                for (int c = 0; c < 5; ++c) {
                    const int gy = gy0 + r, gx = gx0 + c;
                    const bool in = lane_on && gy >= 0 && gy < H && gx >= 0 && gx < W;
                    const unsigned off = in ? (unsigned)(((ci * H + gy) * W + gx) * 4) : 0xfffffff0u;
                    x[ci][r][c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xr, off, 0, 0));
                }
    }

    // Convolution outputs outside the layer's extent must not win a maximum: their sums start from -FLT_MAX
    // instead of 0 (section 3.3: the next layer's padding value in place), which the multiply-adds of finite
    // inputs leave unchanged.
    const float s00 = (lane_on && cy0 < P.H1 && cx0 < P.W1) ? 0.f : -FLT_MAX;
    const float s01 = (lane_on && cy0 < P.H1 && cx0 + 1 < P.W1) ? 0.f : -FLT_MAX;
    const float s10 = (lane_on && cy0 + 1 < P.H1 && cx0 < P.W1) ? 0.f : -FLT_MAX;
    const float s11 = (lane_on && cy0 + 1 < P.H1 && cx0 + 1 < P.W1) ? 0.f : -FLT_MAX;
    const bool out_ok = lane_on && by < P.th && bx < P.tw && py < P.Ho && px < P.Wo;

    const int cout = P.c1.cout;
    const int nbatch = (cout + CB - 1) / CB;
    cfloat *shift_s = (cfloat *)(unsigned long long)P.c1.aff;
    const size_t oplane = (size_t)P.Ho * P.Wo;
    const __amdgpu_buffer_rsrc_t yr = make_rsrc(P.y + ((size_t)n * P.Cy + P.coff1) * oplane,
                                                ((unsigned long long)(P.N - n) * P.Cy - P.coff1) * oplane * 4ull);
    const unsigned own = (unsigned)((py * P.Wo + px) * 4);
    const int lo = P.c1.relu ? 0 : INT_MIN;

    float wa[RS], wb[RS];
    {
        cfloat *wr = (cfloat *)(unsigned long long)P.c1.wp;
#pragma unroll
        for (int t = 0; t < RS; ++t) wa[t] = wr[t];
    }
    static_assert(CB % 2 == 0, "the two filter-row sets alternate");
    for (int b = 0; b < nbatch; ++b) {
        float *buf = lds + (b & 1) * (CB * 3) * nthreads;
        float m_all[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            // The filter row of the NEXT channel (rows are padded to whole 64-byte lines) is requested before this
            // channel's multiply-adds and lands in the other of two sets of scalar registers meanwhile.
            const float (&w16)[RS] = (c % 2 == 0) ? wa : wb;
            float (&wnext)[RS] = (c % 2 == 0) ? wb : wa;
            {
                cfloat *wr = (cfloat *)(unsigned long long)P.c1.wp + (size_t)min(b * CB + c + 1, nbatch * CB - 1) * RS;   // (rows exist up to the next multiple of 16 channels)
#pragma unroll
                for (int t = 0; t < RS; ++t) wnext[t] = wr[t];
            }
            float a00 = s00, a01 = s01, a10 = s10, a11 = s11;
#pragma unroll
            for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
                for (int u = 0; u < 3; ++u)
#pragma unroll
                    for (int v = 0; v < 3; ++v) {
                        const int t = (ci * 3 + u) * 3 + v;
                        const float w = w16[t];
                        a00 = fmaf(x[ci][u][v], w, a00);
                        a01 = fmaf(x[ci][u][v + 2], w, a01);
                        a10 = fmaf(x[ci][u + 2][v], w, a10);
                        a11 = fmaf(x[ci][u + 2][v + 2], w, a11);
                    }
            const float top = fmaxf(a00, a01), left = fmaxf(a00, a10);
            m_all[c] = fmaxf(top, fmaxf(a10, a11));
            // (pins the value here: the compiler otherwise moves the fourth sum behind the barrier, into the branch of
            // the lanes that store, and has to keep or reload the filter rows for it)
            asm volatile("" : "+v"(m_all[c]));
            buf[(c * 3 + 0) * nthreads + tid] = left;
            buf[(c * 3 + 1) * nthreads + tid] = top;
            buf[(c * 3 + 2) * nthreads + tid] = a00;
            __builtin_amdgcn_sched_barrier(0);      // a channel's multiply-adds stay together, its filter row dies here
        }
        __syncthreads();
        if (out_ok) {
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                const int oc = b * CB + c;
                float m = fmaxf(fmaxf(m_all[c], buf[(c * 3 + 0) * nthreads + tid + 1]),
                                fmaxf(buf[(c * 3 + 1) * nthreads + tid + bw], buf[(c * 3 + 2) * nthreads + tid + bw + 1]));
                m += shift_s[oc];
                m = __builtin_bit_cast(float, max(__builtin_bit_cast(int, m), lo));      // ReLU as an integer maximum
                if (oc < cout) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, m), yr, own, oc * (int)oplane * 4, 0);
            }
        }
        // the next batch goes to the other tile; this one is overwritten two batches on, after the barrier in between
    }
}

// Filter of a thin layer: [Cout][row of thin_row_floats(Cin*K*K)] times the per-channel scale, zero past the taps of a
// row and in the rows up to the next multiple of 16 channels; shift likewise.
__global__ void pack_thin_kernel(const float *__restrict__ w, const float *__restrict__ scale,
                                 const float *__restrict__ shift, float *__restrict__ wp, float *__restrict__ aff,
                                 int cout, int taps)
{
    const int rows = (cout + 15) / 16 * 16;
    const int rs = thin_row_floats(taps);
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < rows * rs) {
        const int oc = idx / rs, t = idx - oc * rs;
        wp[idx] = (oc < cout && t < taps) ? w[oc * taps + t] * (scale ? scale[oc] : 1.f) : 0.f;
    }
    if (idx < rows) aff[idx] = (idx < cout && shift) ? shift[idx] : 0.f;
}

}  // namespace xl
