// Thin first layers on the vector ALU (included by kernels.hip).
//
// A convolution with a handful of input channels (the 3-channel stem of an image network) gives the
// matrix cores a reduction of 27 terms: most of a K step is padding, and the layer is bound by moving
// its input and output, not by arithmetic (paper section 2.2: convolutions with few input channels are
// memory-bound).  Here it runs as plain multiply-adds instead:
//   - a lane owns one OUTPUT CHANNEL (64 per wavefront) and keeps that channel's whole filter,
//     Cin * K * K values, in registers for the life of the wavefront;
//   - the input pixels are the same for every lane, so they are not vector data at all: they are read
//     with scalar loads straight from the input tensor (wave-uniform addresses, constant address
//     space) and enter v_fma_f32 as its scalar operand.  No LDS, no staging, no barrier;
//   - a following max pooling (paper Fig. 3b: Layer2 consumes Layer1's output on chip) happens in the
//     same lane: the PK x (PS * (PW - 1) + PK) convolution outputs under one row of PW pooled pixels
//     live in registers, rows shared by two pooled rows are kept, and only pooled values are stored.
//     Bias and ReLU are applied after the maximum (both are monotonic, so the result is bit-identical
//     to applying them to every convolution output first).
// A wavefront works on one item: (image, group of 64 output channels, tile of th x PW pooled pixels).
// Everything but the final store mask is wave-uniform control flow.
//
// BlockParams fields used: x, y, N, Cin, H, W, H1, W1 (convolution output extent), Ho, Wo (block output
// extent), Cy, coff1, c1 (wp: filter as [channel group][Cin*K*K][64 lanes] with the scale folded in,
// aff: shift as [channel group][64 lanes]; stride, pad, relu, cout), P2 (padding of the pooling),
// th (pooled rows per item), tiles_x, tiles_y, csplit (channel groups), nblocks (items).
#pragma once

namespace xl {

constexpr int THIN_PW = THIN_TILE_W;      // pooled (without pooling: convolution) columns per item

template <int CIN, int K, int S, int PK, int PS, int G = 4>
__global__ void __launch_bounds__(256) thin_conv_kernel(const BlockParams P)
{
    constexpr int PW = THIN_PW;
    constexpr int CC = PS * (PW - 1) + PK;          // convolution columns under one row of pooled pixels
    constexpr int T = CIN * K * K;
    constexpr int KEEP = PK > PS ? PK - PS : 0;     // convolution rows two consecutive pooled rows share
    constexpr int NX = S * (G - 1) + K;             // input columns under G convolution pixels
    typedef const float __attribute__((address_space(4))) cfloat;    // read-only, wave-uniform: scalar loads

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int item = __builtin_amdgcn_readfirstlane(logical_block() * (int)(blockDim.x >> 6) + wave);
    if (item >= P.nblocks) return;
    const int tx = item % P.tiles_x;
    int r = item / P.tiles_x;
    const int ty = r % P.tiles_y;
    r /= P.tiles_y;
    const int cg = r % P.csplit;
    const int n = r / P.csplit;

    const int oc = cg * 64 + lane;
    float w[T];
    {
        const float *wp = reinterpret_cast<const float *>(P.c1.wp) + (size_t)cg * T * 64 + lane;
#pragma unroll
        for (int t = 0; t < T; ++t) w[t] = wp[t * 64];
    }
    const float shift = reinterpret_cast<const float *>(P.c1.aff)[cg * 64 + lane];

    const int H = P.H, W = P.W, pad = P.c1.pad;
    const int py0 = ty * P.th, px0 = tx * PW;                   // first pooled pixel of the item
    const int cy0 = py0 * PS - P.P2, cx0 = px0 * PS - P.P2;     // first convolution output under its windows
    const float *xg = P.x + (size_t)n * CIN * H * W;            // this image, for per-lane loads
    cfloat *xn = (cfloat *)(unsigned long long)xg;              // the same, for scalar loads
    const size_t oplane = (size_t)P.Ho * P.Wo;
    const __amdgpu_buffer_rsrc_t yr = make_rsrc(P.y + ((size_t)n * P.Cy + P.coff1) * oplane,
                                                ((unsigned long long)(P.N - n) * P.Cy - P.coff1) * oplane * 4ull);

    // filter value of a run-time channel (the border path loops over channels to stay small)
    auto wsel = [&](int ci, int t) {
        float r = w[t];
#pragma unroll
        for (int c = 1; c < CIN; ++c) r = ci == c ? w[c * K * K + t] : r;
        return r;
    };
    float cv[PK][CC];
    // One row of convolution outputs (without shift and activation); -FLT_MAX where the pooling must not
    // look.  Columns are worked off in groups of G that share one run of input columns per (channel, filter
    // row).  A run that lies inside the image row is read with scalar loads; a run that crosses the
    // row's ends (padding, the ragged last item of a row) is fetched by the first lanes with a bounds
    // check and handed out with v_readlane.
    auto conv_row = [&](float (&out)[CC], int cr) {
        if (cr < 0 || cr >= P.H1) {
#pragma unroll
            for (int c = 0; c < CC; ++c) out[c] = -FLT_MAX;
            return;
        }
        const int gy0 = cr * S - pad;
#pragma unroll
        for (int c0 = 0; c0 < CC; c0 += G) {
            const int gcount = CC - c0 < G ? CC - c0 : G;           // compile-time after unrolling
            const int run = S * (gcount - 1) + K;                   // input columns under the group
            const int cc0 = cx0 + c0;                               // first convolution column of the group
            const int gx0 = cc0 * S - pad;                          // first input column under it
            float acc[G];
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = 0.f;
            // every input element under the group inside the image: all its runs in one burst of scalar loads
            const bool fast = gx0 >= 0 && gx0 + run <= W && gy0 >= 0 && gy0 + K <= H;
            if (fast) {
                cfloat *first = xn + (size_t)gy0 * W + gx0;
                float xr[CIN][K][NX];
#pragma unroll
                for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
                    for (int u = 0; u < K; ++u)
#pragma unroll
                        for (int v = 0; v < NX; ++v)
                            if (v < run) xr[ci][u][v] = first[((size_t)ci * H + u) * W + v];
                __builtin_amdgcn_sched_barrier(0);      // every load of the group in flight before the first use: one wait
#pragma unroll
                for (int ci = 0; ci < CIN; ++ci)
#pragma unroll
                    for (int u = 0; u < K; ++u)
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            if (g >= gcount) continue;
#pragma unroll
                            for (int v = 0; v < K; ++v) acc[g] = fmaf(xr[ci][u][g * S + v], w[(ci * K + u) * K + v], acc[g]);
                        }
            } else if (cc0 + gcount > 0 && cc0 < P.W1) {
                for (int ci = 0; ci < CIN; ++ci) {
#pragma unroll
                    for (int u = 0; u < K; ++u) {
                        const int gy = gy0 + u;
                        if (gy < 0 || gy >= H) continue;           // a row of padding adds nothing
                        const size_t ro = ((size_t)ci * H + gy) * W;
                        const int gx = gx0 + lane;
                        const bool ok = lane < run && gx >= 0 && gx < W;
                        const float t = ok ? xg[ro + (ok ? gx : 0)] : 0.f;
                        float xr[NX];
#pragma unroll
                        for (int v = 0; v < NX; ++v)
                            if (v < run)
                                xr[v] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), v));
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            if (g >= gcount) continue;
#pragma unroll
                            for (int v = 0; v < K; ++v) acc[g] = fmaf(xr[g * S + v], wsel(ci, u * K + v), acc[g]);
                        }
                    }
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (g >= gcount) continue;
                const int cc = cc0 + g;
                out[c0 + g] = (cc >= 0 && cc < P.W1) ? acc[g] : -FLT_MAX;
            }
        }
    };

    // Pooled rows top to bottom.  Pooled row i looks at convolution rows cr0 .. cr0 + PK - 1, the first KEEP
    // of which it shares with the row above: those are moved up, the other PS are computed.  The loop
    // starts one row early (i = -1) to produce the rows the first pooled row would have inherited.
    const int rows = min(P.th, P.Ho - py0);
    const size_t oplane_oc = (size_t)oc * oplane;
    for (int i = (KEEP > 0 ? -1 : 0); i < rows; ++i) {
        const int cr0 = cy0 + i * PS;       // first convolution row under pooled row py0 + i
#pragma unroll
        for (int u = 0; u < KEEP; ++u)
#pragma unroll
            for (int c = 0; c < CC; ++c) cv[u][c] = cv[u + PS][c];
#pragma unroll
        for (int u = KEEP; u < PK; ++u) {
            if (i < 0 && u < PS) continue;          // warm-up: only the rows pooled row 0 inherits
            conv_row(cv[u], cr0 + u);
        }
        if (i < 0) continue;
        // maximum over the window: rows first, then columns
        float cm[CC];
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            float m = cv[0][c];
#pragma unroll
            for (int u = 1; u < PK; ++u) m = fmaxf(m, cv[u][c]);
            cm[c] = m;
        }
        float o[PW];
#pragma unroll
        for (int j = 0; j < PW; ++j) {
            float m = cm[PS * j];
#pragma unroll
            for (int v = 1; v < PK; ++v) m = fmaxf(m, cm[PS * j + v]);
            m += shift;
            o[j] = P.c1.relu ? fmaxf(m, 0.f) : m;
        }
        // a lane stores PW consecutive pixels of its own channel's row
        const int py = py0 + i;
        const unsigned off = (unsigned)((oplane_oc + (size_t)py * P.Wo + px0) * 4);
        if (oc < P.c1.cout) {
            typedef unsigned u32x4 __attribute__((vector_size(16)));
#pragma unroll
            for (int j = 0; j < PW; j += 4) {
                if (px0 + j + 3 < P.Wo) {
                    const f32x4 v4 = {o[j], o[j + 1], o[j + 2], o[j + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v4), yr, off + 4 * j, 0, 0);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (px0 + j + e < P.Wo)
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, o[j + e]), yr, off + 4 * (j + e), 0, 0);
                }
            }
        }
    }
}

// Filter of a thin layer: [Cout][Cin][K][K] -> [channel group of 64][Cin*K*K][lane], times the per-channel
// scale; shift -> [channel group][lane].  Zero for channels past Cout.
__global__ void pack_thin_kernel(const float *__restrict__ w, const float *__restrict__ scale,
                                 const float *__restrict__ shift, float *__restrict__ wp, float *__restrict__ aff,
                                 int cout, int taps)
{
    const int ncg = (cout + 63) / 64;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < ncg * taps * 64) {
        const int lane = idx & 63, t = (idx >> 6) % taps, cg = (idx >> 6) / taps;
        const int oc = cg * 64 + lane;
        wp[idx] = oc < cout ? w[(size_t)oc * taps + t] * (scale ? scale[oc] : 1.f) : 0.f;
    }
    if (idx < ncg * 64) aff[idx] = (idx < cout && shift) ? shift[idx] : 0.f;
}

}  // namespace xl
