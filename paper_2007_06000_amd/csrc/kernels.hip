// HIP kernels of libxl for gfx950 (CDNA4): tiled implicit-GEMM convolution on the
// fp32 matrix cores, with the block's intermediate feature map held in LDS.
//
// Structure of one workgroup (paper section 2.2, Fig. 3b; section 3.2):
//   S1  stage a halo-extended input tile through LDS in channel chunks
//       (global NCHW -> LDS [channel group of 4][row][col][4], zero outside
//       the image), and accumulate layer 1 for every pixel of the
//       halo-extended intermediate tile                      (LD.G, CONV1)
//   S2  epilogue of layer 1 (scale/shift, ReLU) into the LDS tile; positions
//       outside the image are written as the next layer's padding value
//       (section 3.3, padding strategy)                       (ST.S)
//   S3  workgroup barrier (section 3.3)
//   S4  layer 2 from the LDS tile: one or two sibling convolutions (straight,
//       split) or a max pooling                               (LD.S, CONV2)
//   S5  epilogue (scale/shift, shortcut add for merge, ReLU) and store (ST.G)
//
// Implicit GEMM orientation: matrix-core rows are output channels (A operand =
// filter, streamed from global/L2 in a pre-packed lane order), columns are
// pixels of the tile, flattened row-major (B operand = one float4 LDS read per
// lane giving 4 input channels of one pixel and tap).  Accumulator registers
// of a lane therefore hold 4 consecutive output channels of one pixel, which
// is exactly one float4 of the LDS tile layout.
#include <float.h>

#include "xl_internal.h"

namespace xl {

// Development aid: per-workgroup phase timestamps (only in builds with -DXL_PHASE_TIMING).
#ifdef XL_PHASE_TIMING
__device__ unsigned long long g_phase[16 * 8192];
#define XL_PHASE(L, i)                                                        \
    do {                                                                      \
        if (threadIdx.x == 0 && (L) < 8192) {                                 \
            g_phase[(L) * 16 + (i)] = clock64();                              \
            g_phase[(L) * 16 + 8 + (i)] = wall_clock64();                     \
        }                                                                     \
    } while (0)
#else
#define XL_PHASE(L, i) do { } while (0)
#endif

// ----------------------------------------------------------------------------
// matrix-core wrappers
// ----------------------------------------------------------------------------
template <int MF>
struct MM;

template <>
struct MM<32> {
    typedef f32x16 Acc;
    static constexpr int KC = 8, GPS = 2, NQ = 4;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // first output channel (inside the 32-row tile) of accumulator quad q for lane-half `sub`
    static __device__ __forceinline__ int quad_row(int q, int sub) { return q * 8 + sub * 4; }
};

template <>
struct MM<16> {
    typedef f32x4 Acc;
    static constexpr int KC = 16, GPS = 4, NQ = 1;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int quad_row(int, int sub) { return sub * 4; }
};

template <typename Acc>
__device__ __forceinline__ void zero_acc(Acc &a)
{
#pragma unroll
    for (int i = 0; i < (int)(sizeof(Acc) / sizeof(float)); ++i) a[i] = 0.f;
}

// Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2.
// Map hardware block id -> logical id so that consecutive logical ids (tiles of
// one image, which share halo rows and cache lines of the output) land on the
// same XCD.  gridDim.x is a multiple of 8; ids past `nblocks` do nothing.
__device__ __forceinline__ int logical_block()
{
    const int per = gridDim.x >> 3;
    return (blockIdx.x & 7) * per + (blockIdx.x >> 3);
}

// ----------------------------------------------------------------------------
// K loop: acc[r][p] += filter(row tile r) x pixels(pixel tile p) over `nkg` K steps
// ----------------------------------------------------------------------------
template <int MF, int KS, int NRT, int NPT>
__device__ __forceinline__ void conv_accum(typename MM<MF>::Acc (&acc)[NRT][NPT],
                                           const float *src,             // LDS, group 0 of this K range
                                           const int (&off)[NPT],        // per-lane float offset of tap (0,0)
                                           int src_w, int gstride,
                                           const f32x4 *__restrict__ wpl,   // packed filter + lane, K step 0
                                           const int (&rtc)[NRT],        // row tile of each r (clamped)
                                           int nrt, int nkg)
{
    typedef MM<MF> M;
    constexpr int T = KS * KS;
    constexpr int D = 2;        // software pipeline: operands are fetched D (K step, tap) pairs ahead
    const int kstep = T * nrt * 64;
    f32x4 a[D + 1][NRT], b[D + 1][NPT];
    auto fetch = [&](f32x4(&ra)[NRT], f32x4(&rb)[NPT], int kg, int t) {
        const int u = t / KS, v = t % KS;
        const f32x4 *w = wpl + kg * kstep + t * nrt * 64;
#pragma unroll
        for (int r = 0; r < NRT; ++r) ra[r] = w[rtc[r] * 64];
        const float *s = src + kg * (M::GPS * gstride) + (u * src_w + v) * 4;
#pragma unroll
        for (int p = 0; p < NPT; ++p) rb[p] = *(const f32x4 *)(s + off[p]);
    };
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d / T < nkg) fetch(a[d], b[d], d / T, d % T);
    for (int kg = 0; kg < nkg; ++kg) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (kg + (t + D) / T < nkg) fetch(a[D], b[D], kg + (t + D) / T, (t + D) % T);
            __builtin_amdgcn_sched_barrier(0);      // keep the prefetch ahead of this step's matrix ops
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < NRT; ++r)
#pragma unroll
                    for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(a[0][r][j], b[0][p][j], acc[r][p]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int d = 0; d < D; ++d) {
#pragma unroll
                for (int r = 0; r < NRT; ++r) a[d][r] = a[d + 1][r];
#pragma unroll
                for (int p = 0; p < NPT; ++p) b[d][p] = b[d + 1][p];
            }
        }
    }
}

// ----------------------------------------------------------------------------
// Stage 1: stream the input tile through LDS and accumulate layer 1
// ----------------------------------------------------------------------------
template <int MF, int KS, int NRT, int NPT>
__device__ __forceinline__ void stage1(typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                       const float *__restrict__ ximg, int iy0, int ix0,
                                       int rt0, int rt_end, int pt0, int npx, float *lin)
{
    typedef MM<MF> M;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63;
    const int sub = lane / MF, col = lane % MF;
    const int s1 = P.c1.stride;
    const int HW = P.H * P.W;

    int off[NPT];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        int pidx = (pt0 + p) * MF + col;
        pidx = pidx < npx ? pidx : 0;
        const int my = pidx / P.mw, mx = pidx - my * P.mw;
        off[p] = ((my * s1) * P.iw + mx * s1) * 4 + sub * P.in_gstride;
    }
    int rtc[NRT];
#pragma unroll
    for (int r = 0; r < NRT; ++r) rtc[r] = min(rt0 + r, P.c1.nrt - 1);
    const bool active = rt0 < rt_end && pt0 * MF < npx;

    // what this thread stages per chunk: STAGE_ITEMS float4 items (4 channels of one pixel)
    const int plane = P.ih * P.iw;
    const int nitems = P.chunk_kg * M::GPS * plane;
    int pixoff[STAGE_ITEMS], chan[STAGE_ITEMS];
#pragma unroll
    for (int i = 0; i < STAGE_ITEMS; ++i) {
        const int item = i * nthreads + tid;
        const int g = item / plane, rem = item - g * plane;
        const int r = rem / P.iw, c = rem - r * P.iw;
        const int gy = iy0 + r, gx = ix0 + c;
        const bool in = item < nitems && gy >= 0 && gy < P.H && gx >= 0 && gx < P.W;
        pixoff[i] = in ? gy * P.W + gx : -1;
        chan[i] = g * 4;
    }
    f32x4 st[STAGE_ITEMS];
    auto load_chunk = [&](int c0) {
#pragma unroll
        for (int i = 0; i < STAGE_ITEMS; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int cc = c0 + chan[i] + j;
                st[i][j] = (pixoff[i] >= 0 && cc < P.Cin) ? ximg[(size_t)cc * HW + pixoff[i]] : 0.f;
            }
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int i = 0; i < STAGE_ITEMS; ++i) {
            const int item = i * nthreads + tid;
            if (item < nitems) *(f32x4 *)(lin + item * 4) = st[i];
        }
    };

    const f32x4 *wpl = P.c1.wp + lane;
    const int chunk_c = P.chunk_kg * M::KC;
    const int kstep = KS * KS * P.c1.nrt * 64;
    load_chunk(0);
    store_chunk();
    __syncthreads();
    for (int ch = 0; ch < P.nchunks; ++ch) {
        const bool more = ch + 1 < P.nchunks;
        if (more) load_chunk((ch + 1) * chunk_c);
        const int kg0 = ch * P.chunk_kg;
        const int nkg = min(P.chunk_kg, P.c1.nkg - kg0);
        if (active) conv_accum<MF, KS, NRT, NPT>(acc, lin, off, P.iw, P.in_gstride, wpl + kg0 * kstep, rtc, P.c1.nrt, nkg);
        __syncthreads();
        if (more) {
            store_chunk();
            __syncthreads();
        }
    }
}

__device__ __forceinline__ float ld_or(const float *p, int i, float dflt) { return p ? p[i] : dflt; }

// Epilogue of a tile to global memory (S5), also used by the single-layer kernel.
template <int MF, int NRT, int NPT>
__device__ __forceinline__ void store_global(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                             const ConvW &c, int coff, int n, int oy0, int ox0, int tw,
                                             int rt0, int rt_end, int pt0, int npx, const float *sc, int relu_out)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    const size_t plane = (size_t)P.Ho * P.Wo;
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        const int pidx = (pt0 + p) * MF + col;
        const int oy = pidx / tw, ox = pidx - oy * tw;
        const int gy = oy0 + oy, gx = ox0 + ox;
        const bool pv = pidx < npx && gy < P.Ho && gx < P.Wo;
        const size_t pix = (size_t)gy * P.Wo + gx;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            if (rt0 + r >= rt_end) continue;
#pragma unroll
            for (int q = 0; q < M::NQ; ++q) {
                const int cb = (rt0 + r) * MF + M::quad_row(q, sub);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int co = cb + i;
                    if (pv && co < c.cout) {
                        float v = acc[r][p][q * 4 + i] * ld_or(c.scale, co, 1.f) + ld_or(c.shift, co, 0.f);
                        if (c.relu) v = fmaxf(v, 0.f);
                        if (sc) v += sc[((size_t)n * P.Csc + co) * plane + pix];
                        if (relu_out) v = fmaxf(v, 0.f);
                        P.y[((size_t)n * P.Cy + coff + co) * plane + pix] = v;
                    }
                }
            }
        }
    }
}

// Epilogue of layer 1 into the LDS tile (S2).  `fill` is what the next layer
// must see outside the image: 0 for a convolution, -FLT_MAX for max pooling.
template <int MF, int NRT, int NPT>
__device__ __forceinline__ void store_mid(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                          float *mid, int my0, int mx0, int rt0, int rt_end, int pt0, int npx,
                                          float fill)
{
    typedef MM<MF> M;
    const ConvW &c = P.c1;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        const int pidx = (pt0 + p) * MF + col;
        if (pidx >= npx) continue;
        const int my = pidx / P.mw, mx = pidx - my * P.mw;
        const int gy = my0 + my, gx = mx0 + mx;
        const bool inside = gy >= 0 && gy < P.H1 && gx >= 0 && gx < P.W1;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            if (rt0 + r >= rt_end) continue;
#pragma unroll
            for (int q = 0; q < M::NQ; ++q) {
                const int cb = (rt0 + r) * MF + M::quad_row(q, sub);
                f32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int co = cb + i;
                    float z = 0.f;
                    if (co < c.cout) {
                        z = acc[r][p][q * 4 + i] * ld_or(c.scale, co, 1.f) + ld_or(c.shift, co, 0.f);
                        if (c.relu) z = fmaxf(z, 0.f);
                        if (!inside) z = fill;
                    }
                    v[i] = z;
                }
                *(f32x4 *)(mid + (cb >> 2) * P.mid_gstride + pidx * 4) = v;
            }
        }
    }
}

// Stage 2: one (row-tile group, pixel-tile group) item of a convolution read from the LDS tile.
template <int MF, int KS, int NRT, int NPT>
__device__ __forceinline__ void stage2_item(const BlockParams &P, const ConvW &c, int coff, const float *mid, int n,
                                            int oy0, int ox0, int rt0, int rt_end, int pt0, int npx)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    const int d = P.P2 - c.pad;
    int off[NPT];
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        int pidx = (pt0 + p) * MF + col;
        pidx = pidx < npx ? pidx : 0;
        const int oy = pidx / P.tw, ox = pidx - oy * P.tw;
        off[p] = ((oy * P.s2 + d) * P.mw + ox * P.s2 + d) * 4 + sub * P.mid_gstride;
    }
    int rtc[NRT];
#pragma unroll
    for (int r = 0; r < NRT; ++r) rtc[r] = min(rt0 + r, c.nrt - 1);
    typename M::Acc acc[NRT][NPT];
#pragma unroll
    for (int r = 0; r < NRT; ++r)
#pragma unroll
        for (int p = 0; p < NPT; ++p) zero_acc(acc[r][p]);
    conv_accum<MF, KS, NRT, NPT>(acc, mid, off, P.mw, P.mid_gstride, c.wp + lane, rtc, c.nrt, c.nkg);
    store_global<MF, NRT, NPT>(acc, P, c, coff, n, oy0, ox0, P.tw, rt0, rt_end, pt0, npx, P.sc, P.relu_out);
}

// ----------------------------------------------------------------------------
// The block kernel
// ----------------------------------------------------------------------------
template <int KIND, int MF1, int K1, int NRT1, int NPT1, int MF2>
__global__ void __launch_bounds__(MAX_THREADS) block_kernel(const BlockParams P)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int L = logical_block();
    if (L >= P.nblocks) return;
    const int tiles = P.tiles_x * P.tiles_y;
    const int tile = L % tiles;
    const int cs = (L / tiles) % P.csplit;
    const int n = L / (tiles * P.csplit);
    const int ty = tile / P.tiles_x, tx = tile - ty * P.tiles_x;
    const int oy0 = ty * P.th, ox0 = tx * P.tw;

    const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    typedef MM<MF1> M1;

    // tile origins: output -> intermediate (stage-2 window) -> input (stage-1 window)
    const int my0 = (KIND == KIND_SINGLE) ? oy0 : oy0 * P.s2 - P.P2;
    const int mx0 = (KIND == KIND_SINGLE) ? ox0 : ox0 * P.s2 - P.P2;
    const int iy0 = my0 * P.c1.stride - P.c1.pad;
    const int ix0 = mx0 * P.c1.stride - P.c1.pad;

    float *mid = lds;
    float *lin = lds + P.lds_in_off;
    const float *ximg = P.x + (size_t)n * P.Cin * P.H * P.W;

    // ---- S1: layer 1 over the (halo-extended) tile
    const int npx1 = P.mh * P.mw;
    const int wr = wave % P.waves_r1, wp = wave / P.waves_r1;
    const int wg_rt = P.waves_r1 * NRT1;                         // row tiles one workgroup covers in stage 1
    const int rt_base = (KIND == KIND_SINGLE) ? cs * wg_rt : 0;
    const int rt_end1 = min(P.c1.nrt, rt_base + wg_rt);
    const int rt0 = rt_base + wr * NRT1, pt0 = wp * NPT1;
    typename M1::Acc acc[NRT1][NPT1];
#pragma unroll
    for (int r = 0; r < NRT1; ++r)
#pragma unroll
        for (int p = 0; p < NPT1; ++p) zero_acc(acc[r][p]);
    XL_PHASE(L, 0);
    stage1<MF1, K1, NRT1, NPT1>(acc, P, ximg, iy0, ix0, rt0, rt_end1, pt0, npx1, lin);
    XL_PHASE(L, 1);

    if constexpr (KIND == KIND_SINGLE) {
        store_global<MF1, NRT1, NPT1>(acc, P, P.c1, P.coff1, n, oy0, ox0, P.mw, rt0, rt_end1, pt0, npx1, P.sc,
                                      P.relu_out);
        return;
    } else {
        // ---- S2: epilogue of layer 1 into the LDS tile, S3: barrier
        store_mid<MF1, NRT1, NPT1>(acc, P, mid, my0, mx0, rt0, rt_end1, pt0, npx1,
                                   KIND == KIND_POOL ? -FLT_MAX : 0.f);
        __syncthreads();
        XL_PHASE(L, 2);

        if constexpr (KIND == KIND_POOL) {
            // ---- S4/S5: max pooling from the LDS tile; one float4 (4 channels of one pixel) per item
            const int ngroups = (P.c1.cout + 3) >> 2;
            const int npo = P.th * P.tw;
            const size_t plane = (size_t)P.Ho * P.Wo;
            for (int it = threadIdx.x; it < ngroups * npo; it += blockDim.x) {
                const int g = it / npo, pidx = it - g * npo;
                const int oy = pidx / P.tw, ox = pidx - oy * P.tw;
                const int gy = oy0 + oy, gx = ox0 + ox;
                if (gy >= P.Ho || gx >= P.Wo) continue;
                const float *s = mid + g * P.mid_gstride + ((oy * P.s2) * P.mw + ox * P.s2) * 4;
                f32x4 m = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};
                for (int u = 0; u < P.pool_k; ++u)
                    for (int v = 0; v < P.pool_k; ++v) {
                        const f32x4 t = *(const f32x4 *)(s + (u * P.mw + v) * 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[j]);
                    }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int co = g * 4 + j;
                    if (co < P.c1.cout) P.y[((size_t)n * P.Cy + P.coff1 + co) * plane + (size_t)gy * P.Wo + gx] = m[j];
                }
            }
        } else {
            // ---- S4/S5: sibling convolutions from the LDS tile, heavier one first
            constexpr int NRT2 = nrt2_of(MF2), NPT2 = npt2_of(MF2);
            const int npx2 = P.th * P.tw;
            const int nptg = ((npx2 + MF2 - 1) / MF2 + NPT2 - 1) / NPT2;
            int item = wave;
            for (int ci = 0; ci < P.n2; ++ci) {
                const ConvW &c = P.c2[ci];
                const int per = (c.nrt + P.csplit - 1) / P.csplit;           // row tiles of this workgroup
                const int rtb = cs * per, rte = min(c.nrt, rtb + per);
                const int nrtg = rte > rtb ? (rte - rtb + NRT2 - 1) / NRT2 : 0;
                const int nitems = nrtg * nptg;
                for (; item < nitems; item += nwaves) {
                    const int rtg = item / nptg, ptg = item - rtg * nptg;
                    const int r0 = rtb + rtg * NRT2, p0 = ptg * NPT2;
                    if (c.k == 3)
                        stage2_item<MF2, 3, NRT2, NPT2>(P, c, P.coff2[ci], mid, n, oy0, ox0, r0, rte, p0, npx2);
                    else
                        stage2_item<MF2, 1, NRT2, NPT2>(P, c, P.coff2[ci], mid, n, oy0, ox0, r0, rte, p0, npx2);
                }
                item -= nitems;
            }
        }
        __syncthreads();
        XL_PHASE(L, 3);
    }
}

// ----------------------------------------------------------------------------
// launch table
// ----------------------------------------------------------------------------
typedef void (*BlockKernel)(const BlockParams);

static BlockKernel kernel_of(int variant)
{
    switch (variant) {
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2) \
    case ID:                                  \
        return block_kernel<KIND, MF1, K1, NRT1, NPT1, (MF2 == 0 ? 32 : MF2)>;
        XL_VARIANT_LIST(X)
#undef X
    }
    return nullptr;
}

const std::vector<Variant> &variants()
{
    static const std::vector<Variant> v = {
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2) Variant{ID, KIND, MF1, K1, NRT1, NPT1, MF2},
        XL_VARIANT_LIST(X)
#undef X
    };
    return v;
}

hipError_t configure_kernels(int max_lds_bytes)
{
    for (const Variant &v : variants()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel_of(v.id)),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, max_lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_block(int variant, const BlockParams &p, int threads, size_t lds_bytes, hipStream_t s)
{
    BlockKernel k = kernel_of(variant);
    if (!k) return hipErrorInvalidValue;
    const int grid = (p.nblocks + 7) / 8 * 8;
    hipLaunchKernelGGL(k, dim3(grid), dim3(threads), lds_bytes, s, p);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// filter re-layout: [Cout][Cin][K][K] -> [K step][tap][row tile][lane] float4
//   MF = 32: lane l holds cout = rt*32 + l%32, cin = kg*8  + (l/32)*4 + j
//   MF = 16: lane l holds cout = rt*16 + l%16, cin = kg*16 + (l/16)*4 + j
// zero where cout or cin run past the real extent.
// ----------------------------------------------------------------------------
__global__ void pack_filter_kernel(const float *__restrict__ w, f32x4 *__restrict__ wp, int cout, int cin, int k,
                                   int mf, int nkg, int nrt)
{
    const int taps = k * k;
    const long long total = (long long)nkg * taps * nrt * 64;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    long long r = idx >> 6;
    const int rt = (int)(r % nrt);
    r /= nrt;
    const int t = (int)(r % taps);
    const int kg = (int)(r / taps);
    const int o = rt * mf + lane % mf;
    const int sub = lane / mf;
    const int kc = mf == 32 ? 8 : 16;
    f32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int ci = kg * kc + sub * 4 + j;
        v[j] = (o < cout && ci < cin) ? w[((size_t)o * cin + ci) * taps + t] : 0.f;
    }
    wp[idx] = v;
}

hipError_t launch_pack_filter(const float *w, f32x4 *wp, int cout, int cin, int k, int mf, int nkg, int nrt,
                              hipStream_t s)
{
    const long long total = (long long)nkg * k * k * nrt * 64;
    const int threads = 256;
    const int grid = (int)((total + threads - 1) / threads);
    hipLaunchKernelGGL(pack_filter_kernel, dim3(grid), dim3(threads), 0, s, w, wp, cout, cin, k, mf, nkg, nrt);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// element-wise layers of the unfused path
// ----------------------------------------------------------------------------
__global__ void maxpool_kernel(const float *__restrict__ x, float *__restrict__ y, int C, int H, int W, int Ho, int Wo,
                               int k, int stride, int pad, int Cy, int coff, long long total)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int ox = (int)(idx % Wo);
    long long r = idx / Wo;
    const int oy = (int)(r % Ho);
    r /= Ho;
    const int c = (int)(r % C);
    const int n = (int)(r / C);
    const float *xc = x + ((size_t)n * C + c) * H * W;
    float m = -FLT_MAX;
    for (int u = 0; u < k; ++u) {
        const int yy = oy * stride - pad + u;
        if (yy < 0 || yy >= H) continue;
        for (int v = 0; v < k; ++v) {
            const int xx = ox * stride - pad + v;
            if (xx < 0 || xx >= W) continue;
            m = fmaxf(m, xc[(size_t)yy * W + xx]);
        }
    }
    y[(((size_t)n * Cy + coff + c) * Ho + oy) * Wo + ox] = m;
}

hipError_t launch_maxpool(const float *x, float *y, int N, int C, int H, int W, int Ho, int Wo, int k, int stride,
                          int pad, int Cy, int coff, hipStream_t s)
{
    const long long total = (long long)N * C * Ho * Wo;
    if (total == 0) return hipSuccess;
    const int threads = 256;
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)((total + threads - 1) / threads)), dim3(threads), 0, s, x, y, C,
                       H, W, Ho, Wo, k, stride, pad, Cy, coff, total);
    return hipGetLastError();
}

__global__ void add_kernel(const float *__restrict__ a, const float *__restrict__ b, float *__restrict__ y,
                           long long count, int relu)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long n4 = count >> 2;
    if (i < n4) {
        f32x4 va = ((const f32x4 *)a)[i], vb = ((const f32x4 *)b)[i], v;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = va[j] + vb[j];
            if (relu) v[j] = fmaxf(v[j], 0.f);
        }
        ((f32x4 *)y)[i] = v;
    } else if (i == n4) {
        for (long long t = n4 << 2; t < count; ++t) {
            float v = a[t] + b[t];
            y[t] = relu ? fmaxf(v, 0.f) : v;
        }
    }
}

hipError_t launch_add(const float *a, const float *b, float *y, long long count, int relu, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const int threads = 256;
    const long long work = (count >> 2) + 1;
    hipLaunchKernelGGL(add_kernel, dim3((unsigned)((work + threads - 1) / threads)), dim3(threads), 0, s, a, b, y, count,
                       relu);
    return hipGetLastError();
}

// one wavefront per (image, channel): mean over H*W
__global__ void gap_kernel(const float *__restrict__ x, float *__restrict__ y, int NC, int HW)
{
    const int wave = (int)((blockIdx.x * (long long)blockDim.x + threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    if (wave >= NC) return;
    const float *xc = x + (size_t)wave * HW;
    float s = 0.f;
    for (int i = lane; i < HW; i += 64) s += xc[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) y[wave] = s / (float)HW;
}

hipError_t launch_gap(const float *x, float *y, int NC, int HW, hipStream_t s)
{
    if (NC == 0) return hipSuccess;
    const int threads = 256;
    const int wpb = threads / 64;
    hipLaunchKernelGGL(gap_kernel, dim3((NC + wpb - 1) / wpb), dim3(threads), 0, s, x, y, NC, HW);
    return hipGetLastError();
}

}  // namespace xl

#ifdef XL_PHASE_TIMING
extern "C" int xl_debug_read_phases(unsigned long long *host, int count)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(xl::g_phase), sizeof(unsigned long long) * count);
}
#endif
