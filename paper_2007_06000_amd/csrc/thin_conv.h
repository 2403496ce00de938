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
//
// BlockParams fields used: x, y, N, Cin, H, W, H1, W1 (convolution output extent), Ho, Wo (block output
// extent), Cy, coff1, c1 (wp: filter as [Cout rounded up to 16][Cin*K*K] floats with the scale folded
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
            cfloat *wr = wq + (size_t)oc * T;
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
                cfloat *wr = wq + (size_t)(ch * OCB + o) * T;
                float w0[T], w1[T];
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    w0[t] = wr[t];
                    w1[t] = wr[T + t];
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

// Filter of a thin layer: [Cout][Cin*K*K] times the per-channel scale, rows up to the next multiple of 16 zero;
// shift likewise.
__global__ void pack_thin_kernel(const float *__restrict__ w, const float *__restrict__ scale,
                                 const float *__restrict__ shift, float *__restrict__ wp, float *__restrict__ aff,
                                 int cout, int taps)
{
    const int rows = (cout + 15) / 16 * 16;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < rows * taps) {
        const int oc = idx / taps;
        wp[idx] = oc < cout ? w[idx] * (scale ? scale[oc] : 1.f) : 0.f;
    }
    if (idx < rows) aff[idx] = (idx < cout && shift) ? shift[idx] : 0.f;
}

}  // namespace xl
