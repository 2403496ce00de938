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
#include <limits.h>

#include <tuple>
#include <type_traits>

#include "xl_internal.h"

namespace xl {

// ----------------------------------------------------------------------------
// matrix-core wrappers
// ----------------------------------------------------------------------------
// PR = 0: fp32 operands.  PR = 1: every operand is held as two bf16 numbers, hi = bf16(x) and
// lo = bf16(x - hi) (round to nearest), and a product is the sum of three bf16 matrix operations
// hi*hi + hi*lo + lo*hi accumulated in fp32; what is left out is at most 3 * 2^-16 of |a||b|.  One K step
// then covers 16 (MF = 32) or 32 (MF = 16) channels, 8 per lane.  The accumulator layout is the
// same in both modes.
template <int MF, int PR = 0>
struct MM;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <>
struct MM<32, 1> {
    typedef f32x16 Acc;
    static constexpr int KC = 16, GPS = 4, NQ = 4;
    static __device__ __forceinline__ Acc mma(f32x4 a, f32x4 b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

template <>
struct MM<16, 1> {
    typedef f32x4 Acc;
    static constexpr int KC = 32, GPS = 8, NQ = 1;
    static __device__ __forceinline__ Acc mma(f32x4 a, f32x4 b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

template <>
struct MM<32, 0> {
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
struct MM<16, 0> {
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

// max(v, lo) taken on the bit patterns as signed integers, one instruction with `lo` a scalar operand:
// lo = 0 is ReLU (a float with the sign set is a negative integer; -0 becomes +0), lo = INT_MIN the identity.
// So an activation that is switched by a run-time flag costs no compare and no select.
__device__ __forceinline__ float relu_from(float v, int lo)
{
    return __builtin_bit_cast(float, max(__builtin_bit_cast(int, v), lo));
}
__device__ __forceinline__ int relu_bound(int on) { return on ? 0 : INT_MIN; }

// Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2.
// Map hardware block id -> logical id so that consecutive logical ids (tiles of
// one image, which share halo rows and cache lines of the output) land on the
// same XCD.  gridDim.x is a multiple of 8; ids past `nblocks` do nothing.
__device__ __forceinline__ int logical_block()
{
    const int per = gridDim.x >> 3;
    return (blockIdx.x & 7) * per + (blockIdx.x >> 3);
}

// x / d for 0 <= x < 65536 by the multiplier the planner made for d (2^32 / d + 1; 0 stands for d = 1):
// a division by a run-time value costs some 30 vector instructions, and the epilogues need one per
// pixel tile.
__device__ __forceinline__ int fdiv(int x, unsigned magic)
{
    return magic ? (int)__umulhi((unsigned)x, magic) : x;
}

// x / d for any x >= 0 with the same multiplier: the high product is the quotient or one more.
__device__ __forceinline__ int udiv(int x, int d, unsigned magic)
{
    const unsigned q = __umulhi((unsigned)x, magic);
    return magic ? (int)(q - (q * (unsigned)d > (unsigned)x ? 1u : 0u)) : x;
}

// x / d for 0 <= x <= 8 (wave counts), d >= 1: compare and count, scalar instructions when x and d are wave-uniform.
__device__ __forceinline__ int div_upto8(int x, int d)
{
    int q = 0;
#pragma unroll
    for (int k = 1; k <= 8; ++k) q += (x >= k * d) ? 1 : 0;
    return q;
}

// Buffer descriptor over [p, p + bytes) (clamped to 4 GB), raw dword addressing.  Address and size
// are wave-uniform by construction; reading them through the first lane tells the compiler so --
// otherwise every buffer access gets a loop over the distinct descriptor values of the wave.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned long long bytes)
{
    const unsigned long long a = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    const unsigned n = __builtin_amdgcn_readfirstlane((unsigned)(bytes < 0xffffffffull ? bytes : 0xffffffffull));
    return __builtin_amdgcn_make_buffer_rsrc((void *)(((unsigned long long)hi << 32) | lo), (short)0, (int)n, 0x00020000);
}

// ----------------------------------------------------------------------------
// K loop over one staged chunk: acc[r][p] += filter(row tile r) x pixels(pixel tile p).
// Both operands come from LDS: `wsrc` holds the filter chunk as
// [K step][tap][row tile of this workgroup][lane] float4, `bsrc` the pixels as
// [channel group][row][col][4].  Operands of the next (K step, tap) are fetched
// while the matrix cores work on the current one.
// ----------------------------------------------------------------------------
// PX > 0: the pixels come from a planar source, [channel][PX * 64 floats] (only for 1x1 filters):
// `off` then holds the pixel index plus this lane's channel-group offset, and the four channels of a
// K step quarter are four 4-byte reads PX * 64 floats apart (paired by the compiler into two reads
// with 64-dword strides) instead of one 16-byte read.
// JN < 4: only the first JN of the 4 channel slots of every lane hold data (a first layer with at most
// 2 * JN input channels, packed two per slot across the lane halves): the other slots' matrix
// operations would add zeros and are left out.
template <int MF, int KS, int NRT, int NPT, int PX = 0, int JN = 4>
__device__ __forceinline__ void conv_accum(typename MM<MF>::Acc (&acc)[NRT][NPT],
                                           const float *bsrc, const int (&off)[NPT], int src_w, int gstride,
                                           const float *wsrc, const int (&rloc)[NRT], int wg_rt, int nkg)
{
    typedef MM<MF> M;
    constexpr int T = KS * KS;
    const int lane = threadIdx.x & 63;
    f32x4 a[2][NRT], b[2][NPT];
    auto fetch = [&](f32x4(&ra)[NRT], f32x4(&rb)[NPT], int kg, int t) {
        const int u = t / KS, v = t % KS;
        const float *w = wsrc + ((kg * T + t) * wg_rt * 64 + lane) * 4;
#pragma unroll
        for (int r = 0; r < NRT; ++r) ra[r] = *(const f32x4 *)(w + rloc[r] * 256);
        if constexpr (PX == 0) {
            const float *s = bsrc + kg * (M::GPS * gstride) + (u * src_w + v) * 4;
#pragma unroll
            for (int p = 0; p < NPT; ++p) rb[p] = *(const f32x4 *)(s + off[p]);
        } else {
            static_assert(PX == 0 || KS == 1, "planar pixel source is for 1x1 filters");
            const float *s = bsrc + kg * (M::KC * PX * 64);
#pragma unroll
            for (int p = 0; p < NPT; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) rb[p][j] = s[off[p] + j * (PX * 64)];
        }
    };
    // Two operand sets alternate: a step computes from set `cur` while the other one is being fetched;
    // `cur` is a constant once the tap loop is unrolled, so the sets are plain registers.
    static_assert(T % 2 == 1, "filter taps are odd");
    auto step = [&](int cur, int kg, int t) {
        if (t + 1 < T || kg + 1 < nkg) fetch(a[cur ^ 1], b[cur ^ 1], kg + (t + 1) / T, (t + 1) % T);
        __builtin_amdgcn_sched_barrier(0);      // keep the prefetch ahead of this step's matrix ops
#pragma unroll
        for (int j = 0; j < JN; ++j)
#pragma unroll
            for (int r = 0; r < NRT; ++r)
#pragma unroll
                for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(a[cur][r][j], b[cur][p][j], acc[r][p]);
        __builtin_amdgcn_sched_barrier(0);
    };
    fetch(a[0], b[0], 0, 0);
    if constexpr (T == 1) {
        for (int kg = 0; kg < nkg; kg += 2) {
            step(0, kg, 0);
            if (kg + 1 < nkg) step(1, kg + 1, 0);
        }
    } else {
        // with several taps per K step the two sets swap roles once per K step only: one copy there
        // costs less than the registers a loop body of two K steps would take
        for (int kg = 0; kg < nkg; ++kg) {
#pragma unroll
            for (int t = 0; t < T; ++t) step(t & 1, kg, t);
#pragma unroll
            for (int r = 0; r < NRT; ++r) a[0][r] = a[1][r];
#pragma unroll
            for (int p = 0; p < NPT; ++p) b[0][p] = b[1][p];
        }
    }
}

// The same K loop for split-bf16 operands (PR = 1).  Every operand row exists twice in LDS, a hi and
// a lo one: the filter chunk is [K step][tap][row tile][hi, lo][lane] 16 bytes, the pixels are 16-byte
// planes [8-channel group][hi, lo][row][col][8 bf16], `gstride` floats apart (the plane of the
// lane's 8-channel group is part of `off`).  Three matrix operations per tile pair and K step.
template <int MF, int KS, int NRT, int NPT>
__device__ __forceinline__ void conv_accum_b3(typename MM<MF, 1>::Acc (&acc)[NRT][NPT],
                                              const float *bsrc, const int (&off)[NPT], int src_w, int gstride,
                                              const float *wsrc, const int (&rloc)[NRT], int wg_rt, int nkg)
{
    typedef MM<MF, 1> M;
    constexpr int T = KS * KS;
    const int lane = threadIdx.x & 63;
    f32x4 ah[2][NRT], al[2][NRT], bh[2][NPT], bl[2][NPT];
    auto fetch = [&](int set, int kg, int t) {
        const int u = t / KS, v = t % KS;
        const float *w = wsrc + ((kg * T + t) * wg_rt * 128 + lane) * 4;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            ah[set][r] = *(const f32x4 *)(w + rloc[r] * 512);
            al[set][r] = *(const f32x4 *)(w + rloc[r] * 512 + 256);
        }
        const float *s = bsrc + kg * (M::GPS * gstride) + (u * src_w + v) * 4;
#pragma unroll
        for (int p = 0; p < NPT; ++p) {
            bh[set][p] = *(const f32x4 *)(s + off[p]);
            bl[set][p] = *(const f32x4 *)(s + off[p] + gstride);
        }
    };
    static_assert(T % 2 == 1, "filter taps are odd");
    auto step = [&](int cur, int kg, int t) {
        if (t + 1 < T || kg + 1 < nkg) fetch(cur ^ 1, kg + (t + 1) / T, (t + 1) % T);
        __builtin_amdgcn_sched_barrier(0);
        // small terms first; the three products of one tile pair are spread over the other pairs
#pragma unroll
        for (int r = 0; r < NRT; ++r)
#pragma unroll
            for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(al[cur][r], bh[cur][p], acc[r][p]);
#pragma unroll
        for (int r = 0; r < NRT; ++r)
#pragma unroll
            for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(ah[cur][r], bl[cur][p], acc[r][p]);
#pragma unroll
        for (int r = 0; r < NRT; ++r)
#pragma unroll
            for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(ah[cur][r], bh[cur][p], acc[r][p]);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Four or more tile pairs per wave: one operand set only (two would not fit 256 registers); the
    // reads of a step are covered by the other wave of the SIMD and by the step's own 12+ operations.
    if constexpr (NRT * NPT >= 4) {
        for (int kg = 0; kg < nkg; ++kg) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                fetch(0, kg, t);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < NRT; ++r)
#pragma unroll
                    for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(al[0][r], bh[0][p], acc[r][p]);
#pragma unroll
                for (int r = 0; r < NRT; ++r)
#pragma unroll
                    for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(ah[0][r], bl[0][p], acc[r][p]);
#pragma unroll
                for (int r = 0; r < NRT; ++r)
#pragma unroll
                    for (int p = 0; p < NPT; ++p) acc[r][p] = M::mma(ah[0][r], bh[0][p], acc[r][p]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        return;
    }
    fetch(0, 0, 0);
    if constexpr (T == 1) {
        for (int kg = 0; kg < nkg; kg += 2) {
            step(0, kg, 0);
            if (kg + 1 < nkg) step(1, kg + 1, 0);
        }
    } else {
        for (int kg = 0; kg < nkg; ++kg) {
#pragma unroll
            for (int t = 0; t < T; ++t) step(t & 1, kg, t);
#pragma unroll
            for (int r = 0; r < NRT; ++r) { ah[0][r] = ah[1][r]; al[0][r] = al[1][r]; }
#pragma unroll
            for (int p = 0; p < NPT; ++p) { bh[0][p] = bh[1][p]; bl[0][p] = bl[1][p]; }
        }
    }
}

// hi / lo bf16 halves of two floats, packed (first float in the low half of each word)
__device__ __forceinline__ void split_bf16(float a, float b, unsigned &hi, unsigned &lo)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    hi = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{a, b}, bf16x2));
    const float ha = __builtin_bit_cast(float, hi << 16), hb = __builtin_bit_cast(float, hi & 0xffff0000u);
    lo = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{a - ha, b - hb}, bf16x2));
}

// ----------------------------------------------------------------------------
// One pass of a convolution over the tiles this workgroup holds in registers.
// The filter (and, for STAGE_X, the halo-extended input tile) is streamed
// through two LDS buffers in chunks of `chunk_kg` K steps: while the matrix
// cores work on chunk i from one buffer, the global loads of chunk i+1 are in
// flight into registers and are written to the other buffer afterwards; one
// workgroup barrier per chunk.
// ----------------------------------------------------------------------------
struct PassGeom {
    int rt_base;        // first row tile staged by this workgroup
    int wg_rt;          // row tiles staged (= row waves x NRT)
    int wr;             // this wave's position along the row-tile direction
    int chunk_kg;       // K steps per chunk
    int src_w, gstride; // pixel source: tile width, floats per channel group
    int w_off;          // float offset of the filter chunk inside a buffer
    int buf_stride;     // floats between the two buffers
    bool active;        // this wave owns at least one real tile
};

template <int MF, int KS, int NRT, int NPT, bool STAGE_X, int PX = 0, int PR = 0>
__device__ __forceinline__ void conv_pass(typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P, const ConvW &c,
                                          const PassGeom &g, const float *bsrc, const int (&off)[NPT], float *buf,
                                          const float *__restrict__ ximg, unsigned long long x_bytes, int iy0, int ix0)
{
    // ximg: first element of this image of the block input, x_bytes: bytes from there to the end of the tensor
    typedef MM<MF, PR> M;
    static_assert(PR == 0 || PX == 0, "split-bf16 operands are staged through registers");
    constexpr int RW = PR ? 2 : 1;      // 1 KB rows per (K step, tap, row tile) of the filter: hi and lo for PR = 1
    constexpr int T = KS * KS;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    int rloc[NRT];
#pragma unroll
    for (int r = 0; r < NRT; ++r) rloc[r] = g.wr * NRT + r;

    // ---- filter stager: [K step][tap][wg_rt][64] float4 rows of the packed filter go straight from
    // global memory into LDS (LDS-direct 16-byte buffer loads: lane l of a wave writes 16 bytes at the
    // wave-uniform LDS base + 16*l, no staging registers).  One wave instruction moves one
    // (K step, tap, row tile) row of 64 float4; the waves share the rows round-robin.  Row tiles past
    // the filter's last one are skipped: what LDS holds there only feeds accumulator rows that are
    // never stored.  Everything but the per-lane offset is wave-uniform, so a row costs a handful of
    // scalar instructions.  (The buffer form of the load is used, not the global/flat one: the
    // compiler then keeps counting outstanding LDS reads exactly instead of waiting for all of them.)
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves_wg = nthreads >> 6, lane_id = tid & 63;
    const int nkt = c.nkg * T;
    const int f_nrt = c.nrt * RW, f_wg_rt = g.wg_rt * RW, f_base = g.rt_base * RW;     // in 1 KB rows
    const __amdgpu_buffer_rsrc_t wrsrc = make_rsrc(c.wp, (unsigned long long)nkt * f_nrt * 1024ull);
    const int w_lane = (tid & 63) * 16;
    const int w_dkt = div_upto8(nwaves_wg, f_wg_rt), w_drl = nwaves_wg - w_dkt * f_wg_rt;       // row step = nwaves rows
    const int w_kt0 = div_upto8(wave_id, f_wg_rt), w_rl0 = wave_id - w_kt0 * f_wg_rt;
    auto load_w = [&](float *dst, int kg0) {
        const int kts = min(g.chunk_kg * T, nkt - kg0 * T);                     // (K step, tap) rows in this chunk
        const int base = (kg0 * T * f_nrt + f_base) * 1024;                     // byte offset of the chunk's first row
        int kt = w_kt0, rl = w_rl0;
        float *d = dst + wave_id * 256;
        while (kt < kts) {
            if (f_base + rl < f_nrt)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, (__attribute__((address_space(3))) void *)d, 16, w_lane,
                                                         base + (kt * f_nrt + rl) * 1024, 0, 0);
            d += nwaves_wg * 256;
            kt += w_dkt;
            rl += w_drl;
            if (rl >= f_wg_rt) { rl -= f_wg_rt; ++kt; }
        }
    };

    if constexpr (PX > 0) {
        // ---- planar input (1x1 filter, stride 1, no padding: the input tile is the tile of layer 1):
        // the chunk is staged as [channel][PX * 64 floats], each channel holding the ih rows of the tile,
        // iws floats apart, with LDS-direct 16-byte loads, exactly like the filter rows -- no registers,
        // no vector-ALU work.  A wave instruction fills 256 consecutive floats of the chunk; lane l of
        // load i of this wave holds quad Q = (i * nwaves + wave) * 64 + l: channel Q / (PX * 16), and
        // inside the channel row rq / (iws / 4), pixels 4q .. 4q+3 of that row.  Rows start at the first
        // tile column inside the image (xs, see below): a quad that began left of the tensor's first
        // element would read as zeros altogether.  Whatever a quad holds outside the image (rows are
        // clamped into it, a quad may run past its row's end into the next one, or into zeros past the
        // tensor) only feeds pixels of layer 1 outside the image, which the epilogue discards or
        // overwrites.  Cin is a multiple of the K step (planner).
        static_assert(STAGE_X && KS == 1, "planar staging is for stage 1 of 1x1 filters");
        constexpr int QPR = PX * 16;                                   // quads per channel in LDS
        const int HWp = P.H * P.W;
        const int qrow = P.iws >> 2;                                   // quads per tile row
        const int xs = max(0, -ix0);
        const __amdgpu_buffer_rsrc_t xr = make_rsrc(ximg, x_bytes);
        unsigned xvo[PLANAR_SLOTS];
#pragma unroll
        for (int i = 0; i < PLANAR_SLOTS; ++i) {
            const int Q = (i * nwaves_wg + wave_id) * 64 + lane_id;
            const int ch = Q / QPR, rq = Q - ch * QPR;
            const int rr = fdiv(rq, P.rcp_qrow);
            const int r = min(rr, P.ih - 1), q = rq - rr * qrow;
            const int gy = min(max(iy0 + r, 0), P.H - 1);
            xvo[i] = (unsigned)((ch * HWp + gy * P.W + ix0 + xs + 4 * q) * 4);
        }
        auto load_xp = [&](float *dst, int c0) {
            const int loads = min(g.chunk_kg, c.nkg - c0 / M::KC) * (M::KC * QPR / 64);     // wave loads in this chunk
            const int soff = c0 * HWp * 4;
#pragma unroll
            for (int i = 0; i < PLANAR_SLOTS; ++i) {
                const int id = i * nwaves_wg + wave_id;
                if (id < loads)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(dst + id * 256),
                                                             16, xvo[i], soff, 0, 0);
            }
        };
        const int nchunks = (c.nkg + g.chunk_kg - 1) / g.chunk_kg;
        load_w(buf + g.w_off, 0);
        load_xp(buf, 0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        for (int ch = 0; ch < nchunks; ++ch) {
            float *cur = buf + (ch & 1) * g.buf_stride;
            float *nxt = buf + ((ch + 1) & 1) * g.buf_stride;
            const int kg0 = ch * g.chunk_kg;
            if (ch + 1 < nchunks) {
                load_w(nxt + g.w_off, kg0 + g.chunk_kg);
                load_xp(nxt, (kg0 + g.chunk_kg) * M::KC);
            }
            if (g.active)
                conv_accum<MF, KS, NRT, NPT, PX>(acc, cur, off, 0, 0, cur + g.w_off, rloc, g.wg_rt,
                                                 min(g.chunk_kg, c.nkg - kg0));
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
        return;
    }

    // ---- input stager: NCHW -> [group][row][col][4 channels].  A unit is 4 channels x 4 consecutive
    // pixels of one tile row: four 16-byte buffer loads (one per channel), transposed in registers into
    // four float4 LDS writes.  Few, wide loads keep the vector-memory queue short; a wave that has to
    // wait there cannot issue matrix operations either.  The per-lane byte offset of the unit inside
    // the chunk's first channel group is fixed for the whole pass; the channel is a scalar offset; the
    // descriptor starts at the chunk's first channel and ends with the tensor, so whatever a unit
    // touches outside the image (left/right overhang of a row, channels past Cin) is either inside
    // the allocation or reads as zero, and is masked when the unit is written to LDS -- a select
    // right after a load would stall on it.
    typedef unsigned u32x4 __attribute__((vector_size(16)));     // what the 128-bit buffer load returns
    const int HW = P.H * P.W;
    const int plane = P.ih * P.iws;                                // LDS pixels per channel group (rows of iws)
    // Units start at the first tile column that can lie inside the image: a unit that began left of
    // column 0 of the tensor's very first row would have a negative buffer offset, for which the
    // hardware returns zeros for all 16 bytes.  The columns before it are padding and are zero-filled.
    const int xs = max(0, -ix0);
    const int qpr = (P.iw - xs + 3) >> 2;                          // units per tile row
    const int upg = P.ih * qpr;                                    // units per channel group
    const int x_units = STAGE_X ? g.chunk_kg * M::GPS * upg : 0;
    constexpr int NU = STAGE_X ? STAGE_UNITS : 1;
    unsigned xoff[NU];          // byte offset of the unit's first pixel in the group's first channel
    int xdst[NU];               // float offset of that pixel in the LDS chunk
    int xgrp[NU];               // first channel of the unit inside the chunk
    unsigned xmask[NU];         // bit k: pixel k of the unit lies in the tile and inside the image; bits 4, 8: see below
    f32x4 xst[NU][4];
    if constexpr (STAGE_X) {
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            const int u = i * nthreads + tid;
            // (u < 65536; the planner's multipliers cover the tiles that start inside the image and the tx = 0 ones)
            const int e = xs == 0 ? 0 : 1;
            const bool known = xs == 0 || xs == P.xs_left;
            const int gr = known ? fdiv(u, P.rcp_upg[e]) : u / upg, rem = u - gr * upg;
            const int r = known ? fdiv(rem, P.rcp_qpr[e]) : rem / qpr, q = rem - r * qpr;
            const int cc = xs + 4 * q;                              // first tile column of the unit
            const int gy = iy0 + r, gx = ix0 + cc;
            const bool rowok = gy >= 0 && gy < P.H;
            unsigned m = u < x_units ? (q == 0 ? 0x110u : 0x10u) : 0u;      // bit 4: lane owns a unit; bit 8: and zero-fills the row's left padding
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (u < x_units && cc + k < P.iw && rowok && gx + k < P.W) m |= 1u << k;
            }
            xmask[i] = m;
            xgrp[i] = gr * 4;
            // PR = 1: the hi halves of 4-channel group gr go to plane gr & ~1 (the lo halves to the next
            // one), 8 bytes per pixel, after those of group gr - 1 when gr is odd
            xdst[i] = PR ? ((gr & ~1) * plane + r * P.iws + cc) * 4 + (gr & 1) * 2 : (gr * plane + r * P.iws + cc) * 4;
            // lanes without a unit aim past the end of the buffer: the load returns zeros and moves no data
            xoff[i] = u < x_units ? (unsigned)(((gr * 4 * P.H + min(max(gy, 0), P.H - 1)) * P.W + gx) * 4) : 0xfffffff0u;
        }
    }
    __amdgpu_buffer_rsrc_t xrsrc;
    auto load_x = [&](int c0) {                    // chunk whose first channel is c0
        if constexpr (STAGE_X) {
            const unsigned long long skip = (unsigned long long)c0 * HW * 4ull;
            const unsigned long long left = x_bytes > skip ? x_bytes - skip : 0ull;
            xrsrc = make_rsrc((const char *)ximg + skip, left);
#pragma unroll
            for (int i = 0; i < NU; ++i) {
                if (i * nthreads < x_units) {      // uniform: skips unit slots no thread uses
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        xst[i][j] = __builtin_bit_cast(f32x4, (u32x4)__builtin_amdgcn_raw_buffer_load_b128(xrsrc, xoff[i], j * HW * 4, 0));
                }
            }
        }
    };
    // LDS rows are iws = iw rounded up to 4 pixels long, so a unit is always written whole: pixels
    // outside the tile or the image are written as zeros.  A unit of a left-edge tile (xs > 0) may run
    // up to xs pixels past its row's end; there it lands on the next row's left padding (or on the
    // slack behind the chunk), which holds zeros as well.
    auto store_x = [&](float *dst, int c0) {
        if constexpr (STAGE_X) {
            const int nch = P.Cin - c0;            // channels of the chunk that exist (uniform)
            const bool whole = nch >= g.chunk_kg * M::KC;
#pragma unroll
            for (int i = 0; i < NU; ++i) {
                if (i * nthreads < x_units && (xmask[i] & 0x10u)) {
                    if (xs > 0 && (xmask[i] & 0x100u)) {
                        for (int e = 1; e <= xs; ++e) {
                            if constexpr (PR) {
                                *(uint2 *)(dst + xdst[i] - 4 * e) = uint2{0u, 0u};
                                *(uint2 *)(dst + xdst[i] - 4 * e + plane * 4) = uint2{0u, 0u};
                            } else {
                                *(f32x4 *)(dst + xdst[i] - 4 * e) = f32x4{0.f, 0.f, 0.f, 0.f};
                            }
                        }
                    }
                    const int live = whole ? 4 : nch - xgrp[i];        // channels of this unit that exist
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const bool in = (xmask[i] >> k) & 1u;
                        f32x4 v;
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = (in && j < live) ? xst[i][j][k] : 0.f;
                        if constexpr (PR) {
                            uint2 hi, lo;
                            split_bf16(v[0], v[1], hi.x, lo.x);
                            split_bf16(v[2], v[3], hi.y, lo.y);
                            *(uint2 *)(dst + xdst[i] + 4 * k) = hi;
                            *(uint2 *)(dst + xdst[i] + 4 * k + plane * 4) = lo;
                        } else {
                            *(f32x4 *)(dst + xdst[i] + 4 * k) = v;
                        }
                    }
                }
            }
        }
    };

    const int nchunks = (c.nkg + g.chunk_kg - 1) / g.chunk_kg;
    // The input runs two chunks ahead in registers: the units of chunk i + 1 are written to LDS at the
    // start of chunk i, by the few waves that own units, while the other wave of their SIMD already
    // streams matrix operations (vector ALU work squeezed in after a wave's own matrix operations would
    // leave the pipe idle instead); the loads of chunk i + 2 follow into the same registers.
    load_w(buf + g.w_off, 0);
    load_x(0);
    store_x(buf, 0);
    __builtin_amdgcn_s_waitcnt(0);      // this wave's LDS-direct loads have landed
    if (nchunks > 1) load_x(g.chunk_kg * M::KC);
    __syncthreads();
    for (int ch = 0; ch < nchunks; ++ch) {
        float *cur = buf + (ch & 1) * g.buf_stride;
        float *nxt = buf + ((ch + 1) & 1) * g.buf_stride;
        const bool more = ch + 1 < nchunks;
        const int kg0 = ch * g.chunk_kg;
        const int c_next = (kg0 + g.chunk_kg) * M::KC;
        if (more) {
            store_x(nxt, c_next);
            load_w(nxt + g.w_off, kg0 + g.chunk_kg);
            if (ch + 2 < nchunks) load_x(c_next + g.chunk_kg * M::KC);
        }
        const int nkg = min(g.chunk_kg, c.nkg - kg0);
        if (g.active) {
            const float *bs = STAGE_X ? cur : bsrc + kg0 * (M::GPS * g.gstride);
            if constexpr (PR)
                conv_accum_b3<MF, KS, NRT, NPT>(acc, bs, off, g.src_w, g.gstride, cur + g.w_off, rloc, g.wg_rt, nkg);
            else
                conv_accum<MF, KS, NRT, NPT>(acc, bs, off, g.src_w, g.gstride, cur + g.w_off, rloc, g.wg_rt, nkg);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
}

// The per-channel scale and shift (folded BN, bias) cost the epilogues nothing: xl_prepare multiplies
// the scale into the re-laid-out filter (scale * sum(w x) = sum((scale w) x)), and the accumulators start
// from the shift instead of zero (init_acc: the table read overlaps the wait for the first operands, and
// the values live in registers the K loop holds anyway).  An epilogue is activation, masks and stores.

// Accumulators of row tiles rt0 .. rt0 + NRT - 1 start from the per-channel shift: the table xl_prepare
// lays out in accumulator order, [row tile][quad][lane] float4, holds for every lane the 4 consecutive
// output channels of accumulator quad q (0 for channels past Cout).
template <int MF, int NRT, int NPT>
__device__ __forceinline__ void init_acc(typename MM<MF>::Acc (&acc)[NRT][NPT], const ConvW &c, int rt0)
{
    typedef MM<MF> M;
#pragma unroll
    for (int r = 0; r < NRT; ++r) {
        typename M::Acc a;
#pragma unroll
        for (int q = 0; q < M::NQ; ++q) {
            const f32x4 sh = c.aff[(min(rt0 + r, c.nrt - 1) * M::NQ + q) * 64 + (threadIdx.x & 63)];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[q * 4 + i] = sh[i];
        }
#pragma unroll
        for (int p = 0; p < NPT; ++p) acc[r][p] = a;
    }
}

// Epilogue of a tile to global memory (S5), also used by the single-layer kernel.
// Pixel p of the tile sits at (p / vw, p % vw); columns >= tw of the virtual row are padding.
// HAS_SC (merge mode): the shortcut values of one row tile are fetched together before they are used.
// Epilogue into global memory: activation, optional shortcut add, store (the shift is in the accumulators
// already).
template <int MF, int NRT, int NPT, bool HAS_SC>
__device__ __forceinline__ void store_global(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                             const ConvW &c, int coff, int n, int oy0, int ox0, int th, int tw, int vw,
                                             int rt0, int rt_end, int pt0, int relu_out, unsigned rcp_vw)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    // per-image element counts fit 30 bits (checked by the planner): 32-bit offsets from uniform bases
    const int plane = P.Ho * P.Wo;
    float *__restrict__ yn = P.y + ((size_t)n * P.Cy + coff) * plane;
    const float *__restrict__ scn = HAS_SC ? P.sc + (size_t)n * P.Csc * plane : nullptr;
    asm volatile("" ::: "memory");      // keeps the epilogue's address arithmetic out of the K loop's schedule

    // ---- one 4-byte store per accumulator: a lane keeps its pixel, the channel moves through the scalar
    // offset of the buffer instruction (the lane half's +4 channels ride in the lane's own offset), so an
    // element costs one activation and one store, with 32 consecutive pixels of a channel per instruction
    // half.  A vector instruction costs a SIMD about an eighth of a 32x32x2 matrix operation and the two
    // do not overlap, so this beats gathering 16-byte rows through cross-lane moves.
    const unsigned long long ybytes = ((unsigned long long)(P.N - n) * P.Cy - coff) * plane * 4ull;
    const __amdgpu_buffer_rsrc_t yr = make_rsrc(yn, ybytes);
    __amdgpu_buffer_rsrc_t sr = yr;
    if constexpr (HAS_SC) sr = make_rsrc(scn, (unsigned long long)(P.N - n) * P.Csc * plane * 4ull);
    const int lo1 = relu_bound(c.relu), lo2 = relu_bound(relu_out);
    const int lo12 = max(lo1, lo2);
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        const int pidx = (pt0 + p) * MF + col;
        const int oy = fdiv(pidx, rcp_vw), ox = pidx - oy * vw;
        const int gy = oy0 + oy, gx = ox0 + ox;
        const bool pv = oy < th && ox < tw && gy < P.Ho && gx < P.Wo;
        const unsigned voff = (unsigned)((gy * P.Wo + gx + sub * 4 * plane) * 4);
        if (!pv) continue;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            if (rt0 + r >= rt_end) continue;
            const int cb = __builtin_amdgcn_readfirstlane((rt0 + r) * MF);       // first channel of the row tile (wave-uniform)
            // a row tile that lies wholly below Cout (wave-uniform, and the common case) needs no per-element test
            auto row_tile = [&](auto checked) {
                constexpr bool CHECKED = decltype(checked)::value;
                float sv[M::NQ * 4];
                if constexpr (HAS_SC) {
#pragma unroll
                    for (int e = 0; e < M::NQ * 4; ++e) {
                        const int cu = cb + M::quad_row(e >> 2, 0) + (e & 3);            // channel of lane half 0
                        sv[e] = (!CHECKED || cu + sub * 4 < c.cout)
                                    ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(sr, voff, cu * plane * 4, 0))
                                    : 0.f;
                    }
                }
#pragma unroll
                for (int e = 0; e < M::NQ * 4; ++e) {
                    const int cu = cb + M::quad_row(e >> 2, 0) + (e & 3);
                    float v;
                    if constexpr (HAS_SC) v = relu_from(relu_from(acc[r][p][e], lo1) + sv[e], lo2);
                    else v = relu_from(acc[r][p][e], lo12);
                    if (!CHECKED || cu + sub * 4 < c.cout)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), yr, voff, cu * plane * 4, 0);
                }
            };
            if (cb + MF <= c.cout) row_tile(std::false_type{});
            else row_tile(std::true_type{});
        }
    }
}

// Epilogue of a convolution whose only consumer is a global average pooling, with the whole image in
// one workgroup tile: scale / shift / activation, then the mean over the pixels.  Each wave sums its
// accumulators over its pixel tiles and across the lanes that hold different pixels of one channel; the
// waves along the pixel direction meet in LDS (`red`, free once the K loop has ended); one thread per
// channel adds their partial sums in a fixed order and stores the mean.  Called by every wave of the
// workgroup (it contains a barrier); `active` says whether this wave holds real tiles.
template <int MF, int NRT, int NPT>
__device__ __forceinline__ void store_gap(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                          const ConvW &c, int coff, int n, int npx, int rt_base, int wg_rt, int wr,
                                          int wp, int npw, int pt0, bool active, float *red)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    const int rows_wg = wg_rt * MF;
    if (active) {
        asm volatile("" ::: "memory");
        const int lo = max(relu_bound(c.relu), relu_bound(P.relu_out));
        float s[NRT][M::NQ * 4];
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
#pragma unroll
            for (int e = 0; e < M::NQ * 4; ++e) {
                float t = 0.f;
#pragma unroll
                for (int p = 0; p < NPT; ++p) {
                    const float v = relu_from(acc[r][p][e], lo);
                    t += ((pt0 + p) * MF + col < npx) ? v : 0.f;
                }
                // lanes of one `sub` hold the MF pixels of this channel: butterfly over the column bits
#pragma unroll
                for (int m = 1; m < MF; m <<= 1) t += __shfl_xor(t, m, 64);
                s[r][e] = t;
            }
        }
        if (col == 0) {
#pragma unroll
            for (int r = 0; r < NRT; ++r)
#pragma unroll
                for (int e = 0; e < M::NQ * 4; ++e)
                    red[wp * rows_wg + (wr * NRT + r) * MF + M::quad_row(e >> 2, sub) + (e & 3)] = s[r][e];
        }
    } else if (wr * NRT < wg_rt && col == 0) {
        // a wave without real tiles still owns a slot per channel: the sum below reads all of them
#pragma unroll
        for (int r = 0; r < NRT; ++r)
#pragma unroll
            for (int e = 0; e < M::NQ * 4; ++e)
                red[wp * rows_wg + (wr * NRT + r) * MF + M::quad_row(e >> 2, sub) + (e & 3)] = 0.f;
    }
    __syncthreads();
    const float inv = 1.f / (float)npx;
    for (int row = threadIdx.x; row < rows_wg; row += blockDim.x) {
        const int co = rt_base * MF + row;
        if (co < c.cout) {
            float t = 0.f;
            for (int w = 0; w < npw; ++w) t += red[w * rows_wg + row];
            P.y[(size_t)n * P.Cy + coff + co] = t * inv;
        }
    }
}

// Epilogue of layer 1 into the LDS tile (S2).  `fill` is what the next layer
// must see outside the image: 0 for a convolution, -FLT_MAX for max pooling.
// With `add` the result is added to what the tile already holds (the first of two producer layers
// of a merge block, written by this same lane) and `relu_sum` is applied to the sum.
// PR = 1: the tile is written as split-bf16 planes (see conv_accum_b3); `add` reads hi + lo back (exact in fp32).
template <int MF, int NRT, int NPT, int PR = 0>
__device__ __forceinline__ void store_mid(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                          const ConvW &c, float *mid, int my0, int mx0, int rt0, int rt_end, int pt0,
                                          int npx, float fill, bool add = false, bool relu_sum = false)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    asm volatile("" ::: "memory");      // keeps the epilogue's address arithmetic out of the K loop's schedule
    const int lo1 = relu_bound(c.relu), lo2 = relu_bound(relu_sum);
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        const int pidx = (pt0 + p) * MF + col;
        const int my = fdiv(pidx, P.rcp_mw), mx = pidx - my * P.mw;
        const int gy = my0 + my, gx = mx0 + mx;
        const bool inside = gy >= 0 && gy < P.H1 && gx >= 0 && gx < P.W1;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            if (rt0 + r >= rt_end) continue;
            // only a row tile that reaches past Cout (wave-uniform) has channels to blank
            const bool partial = __builtin_amdgcn_readfirstlane((rt0 + r + 1) * MF) > c.cout;
#pragma unroll
            for (int q = 0; q < M::NQ; ++q) {
                const int cb = (rt0 + r) * MF + M::quad_row(q, sub);
                f32x4 v;
                const int gr = cb >> 2;
                float *dst = PR ? mid + (gr & ~1) * P.mid_gstride + pidx * 4 + (gr & 1) * 2
                                : mid + gr * P.mid_gstride + pidx * 4;
                f32x4 old = {0.f, 0.f, 0.f, 0.f};
                if (add && pidx < npx) {
                    if constexpr (PR) {
                        const uint2 oh = *(const uint2 *)dst, ol = *(const uint2 *)(dst + P.mid_gstride);
                        auto up = [](unsigned bits) { return __builtin_bit_cast(float, bits); };
                        old[0] = up(oh.x << 16) + up(ol.x << 16);
                        old[1] = up(oh.x & 0xffff0000u) + up(ol.x & 0xffff0000u);
                        old[2] = up(oh.y << 16) + up(ol.y << 16);
                        old[3] = up(oh.y & 0xffff0000u) + up(ol.y & 0xffff0000u);
                    } else {
                        old = *(const f32x4 *)dst;
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float z = relu_from(acc[r][p][q * 4 + i], lo1);
                    if (add) z = relu_from(z + old[i], lo2);
                    if (!inside) z = fill;
                    if (partial && cb + i >= c.cout) z = 0.f;
                    v[i] = z;
                }
                if constexpr (PR) {
                    uint2 hi, lo;
                    split_bf16(v[0], v[1], hi.x, lo.x);
                    split_bf16(v[2], v[3], hi.y, lo.y);
                    if (pidx < npx) {
                        *(uint2 *)dst = hi;
                        *(uint2 *)(dst + P.mid_gstride) = lo;
                    }
                } else {
                    if (pidx < npx) *(f32x4 *)dst = v;
                }
            }
        }
    }
}

// Epilogue of a stage-2 pass whose result is max-pooled before it leaves the chip (KIND_FUSED2P):
// scale / shift / activation, then into an LDS tile [4-channel group of the pass][row][col][4] of the
// th x tw stage-2 output tile; positions outside the layer's output extent (ragged last tiles, the padding of
// the pooling) get -FLT_MAX, so the pooling windows ignore them.  rl0: this wave's first row tile relative to the pass.
template <int MF, int NRT, int NPT>
__device__ __forceinline__ void store_tile(const typename MM<MF>::Acc (&acc)[NRT][NPT], const BlockParams &P,
                                           const ConvW &c, float *tile, int oy0, int ox0, int rl0, int rt0, int rt_end,
                                           int pt0)
{
    typedef MM<MF> M;
    const int lane = threadIdx.x & 63;
    const int sub = lane / MF, col = lane % MF;
    const int npx = P.th * P.tw;
    asm volatile("" ::: "memory");
    const int lo = relu_bound(c.relu);
#pragma unroll
    for (int p = 0; p < NPT; ++p) {
        const int pidx = (pt0 + p) * MF + col;
        const int oy = fdiv(pidx, P.rcp_vw2), ox = pidx - oy * P.vw2;
        const bool valid = oy < P.th && ox < P.tw;
        const bool inside = oy0 + oy >= 0 && oy0 + oy < P.H2 && ox0 + ox >= 0 && ox0 + ox < P.W2;
#pragma unroll
        for (int r = 0; r < NRT; ++r) {
            if (rt0 + r >= rt_end) continue;
#pragma unroll
            for (int q = 0; q < M::NQ; ++q) {
                const int cl = (rl0 + r) * MF + M::quad_row(q, sub);
                f32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[i] = inside ? relu_from(acc[r][p][q * 4 + i], lo) : -FLT_MAX;
                }
                if (valid) *(f32x4 *)(tile + ((cl >> 2) * npx + oy * P.tw + ox) * 4) = v;
            }
        }
    }
}

// ----------------------------------------------------------------------------
// Depthwise stage 1 (paper Table 1, a.2: a 3x3 convolution with one filter per channel feeding a
// pointwise one).  No reduction over channels, so no matrix cores: the halo-extended input tile of
// all channels is staged as [channel group][row][col][4], then every thread walks (channel group,
// pixel) items, one float4 multiply-add per tap, and writes scale / shift / activation results into
// the LDS tile the pointwise stage reads -- zero where the intermediate lies outside the image.
// Filter: [channel group][tap] float4, scale / shift: [channel group][2] float4 (re-laid out once).
// ----------------------------------------------------------------------------
template <int PR>
__device__ __forceinline__ void depthwise_stage1(const BlockParams &P, float *mid, float *xs, const float *ximg,
                                                 unsigned long long x_bytes, int my0, int mx0, int iy0, int ix0)
{
    const ConvW &c = P.c1;
    const int ncg = (P.Cin + 3) >> 2;
    const int HW = P.H * P.W;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(ximg, x_bytes);
    const int in_px = P.ih * P.iw;
    for (int it = threadIdx.x; it < ncg * in_px; it += blockDim.x) {
        const int g = it / in_px, rem = it - g * in_px;
        const int r = rem / P.iw, cc = rem - r * P.iw;
        const int gy = iy0 + r, gx = ix0 + cc;
        const bool in = gy >= 0 && gy < P.H && gx >= 0 && gx < P.W;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (in) {
            const unsigned off = (unsigned)((g * 4 * HW + gy * P.W + gx) * 4);
#pragma unroll
            for (int j = 0; j < 4; ++j)     // channels past Cin of the last image read as zero (end of the buffer)
                v[j] = (g * 4 + j < P.Cin)
                           ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xr, off, j * HW * 4, 0))
                           : 0.f;
        }
        *(f32x4 *)(xs + (g * P.ih * P.iws + r * P.iws + cc) * 4) = v;
    }
    __syncthreads();
    const int T = c.k * c.k;
    const int mid_px = P.mh * P.mw;
    // the pointwise stage reads whole K steps of 8 or 16 channels: groups past the last real one hold zeros
    const int ncg_all = ((P.Cin + 15) >> 4) << 2;
    for (int it = threadIdx.x; it < ncg_all * mid_px; it += blockDim.x) {
        const int g = it / mid_px, pidx = it - g * mid_px;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        if (g < ncg) {
            const int my = fdiv(pidx, P.rcp_mw), mx = pidx - my * P.mw;
            const float *s = xs + (g * P.ih * P.iws + (my * c.stride) * P.iws + mx * c.stride) * 4;
            const f32x4 *w = c.wp + g * T;
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
            for (int u = 0; u < c.k; ++u)
                for (int v = 0; v < c.k; ++v) {
                    const f32x4 xv = *(const f32x4 *)(s + (u * P.iws + v) * 4);
                    const f32x4 wv = w[u * c.k + v];
#pragma unroll
                    for (int j = 0; j < 4; ++j) a[j] = fmaf(xv[j], wv[j], a[j]);
                }
            const f32x4 sc = c.aff[g * 2], sh = c.aff[g * 2 + 1];
            const int gy = my0 + my, gx = mx0 + mx;
            const bool inside = gy >= 0 && gy < P.H1 && gx >= 0 && gx < P.W1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float t = a[j] * sc[j] + sh[j];
                if (c.relu) t = fmaxf(t, 0.f);
                o[j] = (inside && g * 4 + j < P.Cin) ? t : 0.f;
            }
        }
        if constexpr (PR) {     // split-bf16 planes for the pointwise stage (see conv_accum_b3)
            uint2 hi, lo;
            split_bf16(o[0], o[1], hi.x, lo.x);
            split_bf16(o[2], o[3], hi.y, lo.y);
            float *dst = mid + (g & ~1) * P.mid_gstride + pidx * 4 + (g & 1) * 2;
            *(uint2 *)dst = hi;
            *(uint2 *)(dst + P.mid_gstride) = lo;
        } else {
            *(f32x4 *)(mid + g * P.mid_gstride + pidx * 4) = o;
        }
    }
}

// ----------------------------------------------------------------------------
// The block kernel
// ----------------------------------------------------------------------------
template <int KIND, int MF1, int K1, int NRT1, int NPT1, int MF2, int NRT2, int NPT2, int K2A, int K2B, bool SC, int PX1, int PR = 0>
__global__ void __launch_bounds__(MAX_THREADS, (KIND == KIND_POOL ? 4 : XL_MIN_WAVES)) block_kernel(const BlockParams P)
{
    static_assert(PR == 0 || PX1 == 0, "split-bf16 operands are staged through registers");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int L = logical_block();
    if (L >= P.nblocks) return;
    const int tiles = P.tiles_x * P.tiles_y;
    const int n = udiv(L, tiles * P.csplit, P.rcp_tcs);
    const int in_image = L - n * tiles * P.csplit;
    const int cs = udiv(in_image, tiles, P.rcp_tiles);
    const int tile = in_image - cs * tiles;
    const int ty = udiv(tile, P.tiles_x, P.rcp_tiles_x), tx = tile - ty * P.tiles_x;
    // KIND_FUSED2P: th x tw is the stage-2 tile the pooled pth x ptw output tile needs; neighbours overlap
    const int oy0 = (KIND == KIND_FUSED2P) ? ty * P.pth * P.ps2 - P.pp : ty * P.th;
    const int ox0 = (KIND == KIND_FUSED2P) ? tx * P.ptw * P.ps2 - P.pp : tx * P.tw;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    typedef MM<MF1, PR> M1;
    constexpr int SUBP = PR ? 2 : 1;    // 16-byte planes per lane group of a K step (hi and lo for PR = 1)

    // tile origins: output -> intermediate (stage-2 window) -> input (stage-1 window)
    const int my0 = (KIND == KIND_SINGLE) ? oy0 : oy0 * P.s2 - P.P2;
    const int mx0 = (KIND == KIND_SINGLE) ? ox0 : ox0 * P.s2 - P.P2;
    const int iy0 = my0 * P.c1.stride - P.c1.pad;
    const int ix0 = mx0 * P.c1.stride - P.c1.pad;

    float *mid = lds;
    float *buf = lds + P.lds_buf_off;
    const float *ximg = P.x + (size_t)n * P.Cin * P.H * P.W;

    if constexpr (KIND == KIND_DW) {
        // ---- S1/S2 for a depthwise first layer: vector ALU from a staged input tile into the LDS tile
        depthwise_stage1<PR>(P, mid, buf, ximg, (unsigned long long)(P.N - n) * P.Cin * P.H * P.W * 4ull, my0, mx0, iy0, ix0);
    } else {
    // ---- S1: layer 1 over the (halo-extended) tile
    const int npx1 = P.mh * P.mw;
    PassGeom g1;
    g1.wg_rt = P.waves_r1 * NRT1;
    g1.rt_base = (KIND == KIND_SINGLE) ? cs * g1.wg_rt : 0;
    const int lg_r1 = __builtin_ctz(P.waves_r1);          // wave layouts are powers of two
    g1.wr = wave & (P.waves_r1 - 1);
    g1.chunk_kg = P.chunk_kg;
    g1.src_w = P.iws;
    g1.gstride = P.in_gstride;
    g1.w_off = P.w_off1;
    g1.buf_stride = P.buf_stride;
    const int rt_end1 = min(P.c1.nrt, g1.rt_base + g1.wg_rt);
    const int rt0 = g1.rt_base + g1.wr * NRT1, pt0 = (wave >> lg_r1) * NPT1;
    g1.active = rt0 < rt_end1 && pt0 * MF1 < npx1;
    typename M1::Acc acc[NRT1][NPT1];
    int off1[NPT1];
    {
        const int sub = lane / MF1, col = lane % MF1;
#pragma unroll
        for (int p = 0; p < NPT1; ++p) {
            int pidx = (pt0 + p) * MF1 + col;
            pidx = pidx < npx1 ? pidx : 0;
            const int my = fdiv(pidx, P.rcp_mw), mx = pidx - my * P.mw;
            off1[p] = PX1 > 0 ? my * P.iws + max(mx - max(0, -ix0), 0) + sub * (4 * PX1 * 64)
                              : ((my * P.c1.stride) * P.iws + mx * P.c1.stride) * 4 + sub * SUBP * P.in_gstride;
        }
    }
    init_acc<MF1, NRT1, NPT1>(acc, P.c1, rt0);
    conv_pass<MF1, K1, NRT1, NPT1, true, PX1, PR>(acc, P, P.c1, g1, nullptr, off1, buf, ximg,
                                                  (unsigned long long)(P.N - n) * P.Cin * P.H * P.W * 4ull, iy0, ix0);

    if constexpr (KIND == KIND_SINGLE) {
        if (P.gap) {
            store_gap<MF1, NRT1, NPT1>(acc, P, P.c1, P.coff1, n, npx1, g1.rt_base, g1.wg_rt, g1.wr, wave >> lg_r1,
                                       nwaves >> lg_r1, pt0, g1.active, buf);
            return;
        }
        if (g1.active)
            store_global<MF1, NRT1, NPT1, false>(acc, P, P.c1, P.coff1, n, oy0, ox0, P.mh, P.mw, P.mw, rt0, rt_end1, pt0,
                                                 P.relu_out, P.rcp_mw);
        return;
    } else {
        // ---- S2: epilogue of layer 1 into the LDS tile
        store_mid<MF1, NRT1, NPT1, (KIND == KIND_POOL ? 0 : PR)>(acc, P, P.c1, mid, my0, mx0, rt0, rt_end1, pt0, npx1,
                                                                 KIND == KIND_POOL ? -FLT_MAX : 0.f);
        if constexpr (KIND == KIND_FUSED2 && K1 == 1 && K2A == 1 && K2B == 0 && !SC) {
            if (P.n1 == 2) {
                // second producer of a merge block (paper Fig. 4c): same input, same geometry, its own
                // filter; its result is added to the first one's in the LDS tile
                init_acc<MF1, NRT1, NPT1>(acc, P.c1b, rt0);
                conv_pass<MF1, K1, NRT1, NPT1, true, PX1, PR>(acc, P, P.c1b, g1, nullptr, off1, buf, ximg,
                                                         (unsigned long long)(P.N - n) * P.Cin * P.H * P.W * 4ull, iy0, ix0);
                store_mid<MF1, NRT1, NPT1, PR>(acc, P, P.c1b, mid, my0, mx0, rt0, rt_end1, pt0, npx1, 0.f, true,
                                               P.relu_mid != 0);
            }
        }
    }
    }
    if constexpr (KIND != KIND_SINGLE) {
        // ---- S3: barrier between producing and consuming the LDS tile
        __syncthreads();

        if constexpr (KIND == KIND_POOL) {
            // ---- S4/S5: max pooling from the LDS tile; one float4 (4 channels of one pixel) per item
            const int ngroups = (P.c1.cout + 3) >> 2;
            const int npo = P.th * P.tw;
            const size_t plane = (size_t)P.Ho * P.Wo;
            for (int it = threadIdx.x; it < ngroups * npo; it += blockDim.x) {
                const int gq = udiv(it, npo, P.rcp_npo), pidx = it - gq * npo;
                const int oy = fdiv(pidx, P.rcp_pw), ox = pidx - oy * P.tw;
                const int gy = oy0 + oy, gx = ox0 + ox;
                if (gy >= P.Ho || gx >= P.Wo) continue;
                const float *s = mid + gq * P.mid_gstride + ((oy * P.s2) * P.mw + ox * P.s2) * 4;
                f32x4 m = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};
                if (P.pool_k == 3) {        // the usual window, unrolled: nine reads in flight together
                    f32x4 t[9];
#pragma unroll
                    for (int u = 0; u < 3; ++u)
#pragma unroll
                        for (int v = 0; v < 3; ++v) t[u * 3 + v] = *(const f32x4 *)(s + (u * P.mw + v) * 4);
#pragma unroll
                    for (int k = 0; k < 9; ++k)
#pragma unroll
                        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[k][j]);
                } else {
                    for (int u = 0; u < P.pool_k; ++u)
                        for (int v = 0; v < P.pool_k; ++v) {
                            const f32x4 t = *(const f32x4 *)(s + (u * P.mw + v) * 4);
#pragma unroll
                            for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[j]);
                        }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int co = gq * 4 + j;
                    if (co < P.c1.cout) P.y[((size_t)n * P.Cy + P.coff1 + co) * plane + (size_t)gy * P.Wo + gx] = m[j];
                }
            }
        } else {
            // ---- S4/S5: sibling convolutions from the LDS tile, heavier one first.  Every pass covers
            // (row waves x NRT2) row tiles by (pixel waves x NPT2) pixel tiles; all waves stream the
            // same filter chunks.
            const int sub = lane / MF2, col = lane % MF2;
            const int npt2 = (P.th * P.vw2 + MF2 - 1) / MF2;
            const int lg_r2 = __builtin_ctz(P.waves_r2);
            const int wr2 = wave & (P.waves_r2 - 1), wp2 = wave >> lg_r2;
            const int wg_pt2 = (nwaves >> lg_r2) * NPT2;
            auto run_conv = [&](auto ks_tag, const ConvW &c, int coff, int chunk_kg2) {
                constexpr int KS2 = decltype(ks_tag)::value;
                const int per = udiv(c.nrt + P.csplit - 1, P.csplit, P.rcp_csplit);     // row tiles of this workgroup
                const int rtb = cs * per, rte = min(c.nrt, rtb + per);
                PassGeom g2;
                g2.wg_rt = P.waves_r2 * NRT2;
                g2.wr = wr2;
                g2.chunk_kg = chunk_kg2;
                g2.src_w = P.mw;
                g2.gstride = P.mid_gstride;
                g2.w_off = 0;
                g2.buf_stride = P.buf_stride;
                const int d = P.P2 - c.pad;
                for (int rp = rtb; rp < rte; rp += g2.wg_rt) {
                    for (int pp = 0; pp < npt2; pp += wg_pt2) {
                        g2.rt_base = rp;
                        const int r0 = rp + wr2 * NRT2, p0 = pp + wp2 * NPT2;
                        g2.active = r0 < rte && p0 < npt2;
                        typename MM<MF2>::Acc acc2[NRT2][NPT2];
                        int off2[NPT2];
                        init_acc<MF2, NRT2, NPT2>(acc2, c, r0);
#pragma unroll
                        for (int p = 0; p < NPT2; ++p) {
                            const int pidx = (p0 + p) * MF2 + col;
                            const int oyu = fdiv(pidx, P.rcp_vw2);
                            const int oy = min(oyu, P.th - 1), ox = min(pidx - oyu * P.vw2, P.tw - 1);
                            off2[p] = ((oy * P.s2 + d) * P.mw + ox * P.s2 + d) * 4 + sub * SUBP * P.mid_gstride;
                        }
                        conv_pass<MF2, KS2, NRT2, NPT2, false, 0, PR>(acc2, P, c, g2, mid, off2, buf, nullptr, 0ull, 0, 0);
                        if constexpr (KIND == KIND_FUSED2P) {
                            // the pass covers every pixel of the tile (planner): its result goes to an LDS tile
                            // over the staging buffers, which no wave reads any more, and is pooled from there
                            if (g2.active)
                                store_tile<MF2, NRT2, NPT2>(acc2, P, c, buf, oy0, ox0, wr2 * NRT2, r0, rte, p0);
                            __syncthreads();
                            const int ngr = (min(rte - rp, g2.wg_rt) * MF2) >> 2;
                            const int npo = P.pth * P.ptw, npx2 = P.th * P.tw;
                            const size_t plane = (size_t)P.Ho * P.Wo;
                            for (int it = threadIdx.x; it < ngr * npo; it += blockDim.x) {
                                const int gq = udiv(it, npo, P.rcp_npo), pidx = it - gq * npo;
                                const int py = fdiv(pidx, P.rcp_pw), px = pidx - py * P.ptw;
                                const int gy = ty * P.pth + py, gx = tx * P.ptw + px;
                                if (gy >= P.Ho || gx >= P.Wo) continue;
                                const float *sp = buf + (gq * npx2 + (py * P.ps2) * P.tw + px * P.ps2) * 4;
                                f32x4 m = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};
                                if (P.pool_k == 3) {        // the usual window, unrolled: nine reads in flight together
                                    f32x4 t[9];
#pragma unroll
                                    for (int u = 0; u < 3; ++u)
#pragma unroll
                                        for (int v = 0; v < 3; ++v) t[u * 3 + v] = *(const f32x4 *)(sp + (u * P.tw + v) * 4);
#pragma unroll
                                    for (int k = 0; k < 9; ++k)
#pragma unroll
                                        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[k][j]);
                                } else {
                                    for (int u = 0; u < P.pool_k; ++u)
                                        for (int v = 0; v < P.pool_k; ++v) {
                                            const f32x4 t = *(const f32x4 *)(sp + (u * P.tw + v) * 4);
#pragma unroll
                                            for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[j]);
                                        }
                                }
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int co = rp * MF2 + gq * 4 + j;
                                    if (co < c.cout) P.y[((size_t)n * P.Cy + coff + co) * plane + (size_t)gy * P.Wo + gx] = m[j];
                                }
                            }
                            __syncthreads();
                        } else if (g2.active)
                            store_global<MF2, NRT2, NPT2, SC>(acc2, P, c, coff, n, oy0, ox0, P.th, P.tw, P.vw2, r0, rte,
                                                              p0, P.relu_out, P.rcp_vw2);
                    }
                }
            };
            run_conv(std::integral_constant<int, K2A>{}, P.c2[0], P.coff2[0], P.chunk_kg2[0]);
            if constexpr (K2B != 0) run_conv(std::integral_constant<int, K2B>{}, P.c2[1], P.coff2[1], P.chunk_kg2[1]);
        }
    }
}

// ----------------------------------------------------------------------------
// conv -> max pooling over a stream of tiles (KIND_POOLS).  For a first layer whose whole reduction
// fits one chunk (a few input channels: the stem of an image network) a workgroup's life in
// block_kernel is one long dependency chain: input latency, a short K loop, epilogue, pooling, stores.
// Here a workgroup stays resident and walks tiles L, L + gridDim, ...: the filter is brought to LDS
// once, and the input units of the next tile are requested before the matrix work of the current one,
// so their latency hides behind K loop, epilogue and pooling.  Three barriers per tile:
//   units -> LDS | barrier | request next tile's units, K loop, epilogue -> LDS tile | barrier |
//   pooling -> HBM            (the next tile's "units -> LDS" follows; the first barrier of that tile
//   separates it from this tile's K loop reads, the second from this tile's pooling reads)
// LDS: [intermediate tile][input chunk][filter].  Geometry and parameters as in block_kernel.
// ----------------------------------------------------------------------------
// JN < 4 (MF1 = 32, at most 2 * JN input channels): channel c sits in lane half c % 2, slot c / 2, in
// the staged input as in the filter, and conv_accum skips the empty slots.
template <int MF1, int K1, int NRT1, int NPT1, int JN>
__global__ void __launch_bounds__(MAX_THREADS, 4) pool_stream_kernel(const BlockParams P)
{
    typedef MM<MF1> M1;
    typedef unsigned u32x4 __attribute__((vector_size(16)));
    constexpr int T = K1 * K1;
    static_assert(STAGE_UNITS == 1, "every thread of the stream kernel stages exactly one input unit per tile");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *mid = lds;
    float *xbuf = lds + P.lds_buf_off;
    float *wbuf = xbuf + P.w_off1;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int tiles = P.tiles_x * P.tiles_y;
    const int HW = P.H * P.W;
    const int npx1 = P.mh * P.mw;

    // ---- the whole filter, once
    {
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        const __amdgpu_buffer_rsrc_t wr = make_rsrc(P.c1.wp, (unsigned long long)P.c1.nkg * T * P.c1.nrt * 1024ull);
        const int wg_rt = P.waves_r1 * NRT1;
        const int rows = P.c1.nkg * T * wg_rt;
        for (int row = wave_u; row < rows; row += nwaves) {
            const int kt = row / wg_rt, rl = row - kt * wg_rt;
            if (rl < P.c1.nrt)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void *)(wbuf + row * 256), 16,
                                                         lane * 16, (kt * P.c1.nrt + rl) * 1024, 0, 0);
        }
    }

    // ---- per-wave tile assignment inside a workgroup tile: as in block_kernel
    const int wg_rt = P.waves_r1 * NRT1;
    const int wr = wave % P.waves_r1;
    const int rt_end1 = min(P.c1.nrt, wg_rt);
    const int rt0 = wr * NRT1, pt0 = (wave / P.waves_r1) * NPT1;
    const bool active = rt0 < rt_end1 && pt0 * MF1 < npx1;
    int rloc[NRT1], off1[NPT1];
#pragma unroll
    for (int r = 0; r < NRT1; ++r) rloc[r] = wr * NRT1 + r;
    {
        const int sub = lane / MF1, col = lane % MF1;
#pragma unroll
        for (int p = 0; p < NPT1; ++p) {
            int pidx = (pt0 + p) * MF1 + col;
            pidx = pidx < npx1 ? pidx : 0;
            const int my = fdiv(pidx, P.rcp_mw), mx = pidx - my * P.mw;
            off1[p] = ((my * P.c1.stride) * P.iws + mx * P.c1.stride) * 4 + sub * P.in_gstride;
        }
    }

    // ---- input units of one tile (4 channels x 4 pixels, see conv_pass): one per lane
    const int plane = P.ih * P.iws;
    unsigned xoff = 0, xmask = 0;
    int xdst = 0, xgrp = 0, xs = 0;
    f32x4 xst[4];
    __amdgpu_buffer_rsrc_t xr;
    // Which unit a lane owns depends on the tile only through xs (columns of padding left of the image:
    // tiles of the first column); the two decompositions are made once, not per tile.
    struct UnitPos { int gr, r, q, x_units; };
    auto unit_pos = [&](int xs_) {
        const int qpr = (P.iw - xs_ + 3) >> 2;
        const int upg = P.ih * qpr;
        UnitPos up;
        up.x_units = P.chunk_kg * M1::GPS * upg;             // the one chunk: every K step of the layer
        up.gr = tid / upg;
        const int rem = tid - up.gr * upg;
        up.r = rem / qpr;
        up.q = rem - up.r * qpr;
        return up;
    };
    const int xs_edge = max(0, (P.P2 * P.c1.stride) + P.c1.pad);       // xs of the tiles with tx = 0
    const UnitPos up_in = unit_pos(0), up_edge = unit_pos(xs_edge);
    auto request = [&](int L) {         // descriptor, per-lane unit and loads for tile L
        const int tile = L % tiles, n = L / tiles;
        const int ty = tile / P.tiles_x, tx = tile - ty * P.tiles_x;
        const int iy0 = (ty * P.th * P.s2 - P.P2) * P.c1.stride - P.c1.pad;
        const int ix0 = (tx * P.tw * P.s2 - P.P2) * P.c1.stride - P.c1.pad;
        xs = max(0, -ix0);
        const UnitPos up = xs == 0 ? up_in : (xs == xs_edge ? up_edge : unit_pos(xs));
        const int x_units = up.x_units;
        const int u = tid;
        const int gr = up.gr, r = up.r, q = up.q;
        const int cc = xs + 4 * q;
        const int gy = iy0 + r, gx = ix0 + cc;
        const bool rowok = gy >= 0 && gy < P.H;
        unsigned m = u < x_units ? (q == 0 ? 0x110u : 0x10u) : 0u;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            if (u < x_units && cc + kk < P.iw && rowok && gx + kk < P.W) m |= 1u << kk;
        xmask = m;
        xgrp = gr * 4;
        xdst = (gr * plane + r * P.iws + cc) * 4;
        // lanes without a unit aim past the end of the buffer: the load returns zeros and moves no data
        const int first_ch = JN < 4 ? gr : gr * 4;                   // channel of slot 0 of this unit
        xoff = u < x_units ? (unsigned)(((first_ch * P.H + min(max(gy, 0), P.H - 1)) * P.W + gx) * 4) : 0xfffffff0u;
        xr = make_rsrc(P.x + (size_t)n * P.Cin * HW, (unsigned long long)(P.N - n) * P.Cin * HW * 4ull);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < JN)
                xst[j] = __builtin_bit_cast(f32x4, (u32x4)__builtin_amdgcn_raw_buffer_load_b128(xr, xoff, (JN < 4 ? 2 * j : j) * HW * 4, 0));
            else
                xst[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto deposit = [&]() {              // the requested units -> LDS, masked (pixels outside the image, channels past Cin)
        if (xmask & 0x10u) {
            if (xs > 0 && (xmask & 0x100u)) {
                for (int e = 1; e <= xs; ++e) *(f32x4 *)(xbuf + xdst - 4 * e) = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // slot j holds channel xgrp + j, or with two channels per slot pair (xgrp / 4) + 2 * j
            const int live = JN < 4 ? (P.Cin - (xgrp >> 2) + 1) / 2 : P.Cin - xgrp;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bool in = (xmask >> kk) & 1u;
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = (in && j < live) ? xst[j][kk] : 0.f;
                *(f32x4 *)(xbuf + xdst + 4 * kk) = v;
            }
        }
    };

    // ---- what the epilogue and the pooling need that does not change from tile to tile
    const int sub1 = lane / MF1, col1 = lane % MF1;
    // the shift the accumulators start from stays in registers across tiles when that fits the 128
    // registers of this kernel
    constexpr bool KEEP_AFFINE = NRT1 == 1 && (JN < 4 || MF1 == 16);
    typename M1::Acc acc_init[NRT1][1];
    if constexpr (KEEP_AFFINE) init_acc<MF1, NRT1, 1>(acc_init, P.c1, rt0);
    int e_my[NPT1], e_mx[NPT1], e_pidx[NPT1];
#pragma unroll
    for (int p = 0; p < NPT1; ++p) {
        e_pidx[p] = (pt0 + p) * MF1 + col1;
        e_my[p] = fdiv(e_pidx[p], P.rcp_mw);
        e_mx[p] = e_pidx[p] - e_my[p] * P.mw;
    }
    const int ngroups = (P.c1.cout + 3) >> 2;
    const int npo = P.th * P.tw;
    const size_t oplane = (size_t)P.Ho * P.Wo;
    // first pooling item of this thread (the usual case: no more items than threads)
    const int i_gq = tid / npo, i_pidx = tid - i_gq * npo;
    const int i_oy = i_pidx / P.tw, i_ox = i_pidx - i_oy * P.tw;
    const float *i_sp = mid + i_gq * P.mid_gstride + ((i_oy * P.s2) * P.mw + i_ox * P.s2) * 4;

    const int first = logical_block();
    if (first >= P.nblocks) return;     // uniform per workgroup
    request(first);
    for (int L = first; L < P.nblocks; L += gridDim.x) {
        const int tile = L % tiles, n = L / tiles;
        const int ty = tile / P.tiles_x, tx = tile - ty * P.tiles_x;
        const int oy0 = ty * P.th, ox0 = tx * P.tw;
        const int my0 = oy0 * P.s2 - P.P2, mx0 = ox0 * P.s2 - P.P2;
        deposit();
        __builtin_amdgcn_s_waitcnt(0);          // first tile: this wave's filter rows have landed
        __syncthreads();
        if (L + (int)gridDim.x < P.nblocks) request(L + gridDim.x);
        typename M1::Acc acc[NRT1][NPT1];
        if constexpr (KEEP_AFFINE) {
#pragma unroll
            for (int p = 0; p < NPT1; ++p)
#pragma unroll
                for (int r = 0; r < NRT1; ++r) acc[r][p] = acc_init[r][0];
        } else {
            init_acc<MF1, NRT1, NPT1>(acc, P.c1, rt0);
        }
        if (active)
            conv_accum<MF1, K1, NRT1, NPT1, 0, JN>(acc, xbuf, off1, P.iws, P.in_gstride, wbuf, rloc, wg_rt, P.c1.nkg);
        // epilogue into the LDS tile (store_mid with the tile-independent parts taken from above)
#pragma unroll
        for (int p = 0; p < NPT1; ++p) {
            const int gy = my0 + e_my[p], gx = mx0 + e_mx[p];
            const bool inside = gy >= 0 && gy < P.H1 && gx >= 0 && gx < P.W1;
#pragma unroll
            for (int r = 0; r < NRT1; ++r) {
                if (rt0 + r >= rt_end1) continue;
#pragma unroll
                for (int q = 0; q < M1::NQ; ++q) {
                    const int cb = (rt0 + r) * MF1 + M1::quad_row(q, sub1);
                    f32x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float z = acc[r][p][q * 4 + i];
                        if (P.c1.relu) z = fmaxf(z, 0.f);
                        if (!inside) z = -FLT_MAX;
                        if (cb + i >= P.c1.cout) z = 0.f;
                        v[i] = z;
                    }
                    if (e_pidx[p] < npx1) *(f32x4 *)(mid + (cb >> 2) * P.mid_gstride + e_pidx[p] * 4) = v;
                }
            }
        }
        __syncthreads();
        // pooling from the LDS tile; one float4 (4 channels of one pixel) per item
        const __amdgpu_buffer_rsrc_t yr = make_rsrc(P.y + (size_t)n * P.Cy * oplane, (unsigned long long)(P.N - n) * P.Cy * oplane * 4ull);
        for (int it = tid; it < ngroups * npo; it += nthreads) {
            int gq = i_gq, oy = i_oy, ox = i_ox;
            const float *sp = i_sp;
            if (it != tid) {
                gq = it / npo;
                const int pidx = it - gq * npo;
                oy = pidx / P.tw;
                ox = pidx - oy * P.tw;
                sp = mid + gq * P.mid_gstride + ((oy * P.s2) * P.mw + ox * P.s2) * 4;
            }
            const int gy = oy0 + oy, gx = ox0 + ox;
            if (gy >= P.Ho || gx >= P.Wo) continue;
            f32x4 m = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};
            if (P.pool_k == 3) {        // the usual window, unrolled: nine reads in flight together
                f32x4 t[9];
#pragma unroll
                for (int u = 0; u < 3; ++u)
#pragma unroll
                    for (int v = 0; v < 3; ++v) t[u * 3 + v] = *(const f32x4 *)(sp + (u * P.mw + v) * 4);
#pragma unroll
                for (int k = 0; k < 9; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[k][j]);
            } else {
                for (int u = 0; u < P.pool_k; ++u)
                    for (int v = 0; v < P.pool_k; ++v) {
                        const f32x4 t = *(const f32x4 *)(sp + (u * P.mw + v) * 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) m[j] = fmaxf(m[j], t[j]);
                    }
            }
            // 32-bit offsets from the image's first element (per-image element counts fit 30 bits: planner)
            const unsigned vo = (unsigned)(((P.coff1 + gq * 4) * (int)oplane + gy * P.Wo + gx) * 4);
            const float mv[4] = {m[0], m[1], m[2], m[3]};     // (a bit cast of a vector element picks element 0)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (gq * 4 + j < P.c1.cout)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, mv[j]), yr, vo, j * (int)oplane * 4, 0);
            }
        }
    }
}

}  // namespace xl
#ifndef XL_TU_B3
#include "thin_conv.h"
#endif
namespace xl {

// ----------------------------------------------------------------------------
// launch table
// ----------------------------------------------------------------------------
// Launches through hipLaunchKernel, whose return value is the status of this launch alone (the
// "last error" of the runtime may hold a failure of the caller's own earlier calls).
template <typename... Params, typename... Args>
static hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args)
{
    std::tuple<Params...> values{static_cast<Params>(args)...};
    void *argv[sizeof...(Params)];
    int i = 0;
    std::apply([&](auto &...v) { ((argv[i++] = (void *)&v), ...); }, values);
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds, s);
}

// This file is compiled twice: once for the fp32 variants and everything else, and once with
// XL_TU_B3 defined for the split-bf16 variants alone (the two halves build in parallel).
typedef void (*BlockKernel)(const BlockParams);
BlockKernel kernel_of_b3(int variant);

#ifdef XL_TU_B3
BlockKernel kernel_of_b3(int variant)
{
    switch (variant) {
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1)                                 \
    case ID:                                                                                                 \
        return block_kernel<KIND, MF1, K1, NRT1, NPT1, (MF2 == 0 ? 32 : MF2), (NRT2 == 0 ? 1 : NRT2),        \
                            (NPT2 == 0 ? 1 : NPT2), (K2A == 0 ? 1 : K2A), K2B, (SC != 0), PX1, 1>;
        XL_VARIANT_LIST_B3(X)
#undef X
    }
    return nullptr;
}
#else
template <int KIND, int MF1, int K1, int NRT1, int NPT1, int MF2, int NRT2, int NPT2, int K2A, int K2B, bool SC, int PX1>
static BlockKernel select_kernel()
{
    if constexpr (KIND == KIND_POOLS)
        return pool_stream_kernel<MF1, K1, NRT1, NPT1, (PX1 < 0 ? -PX1 : 4)>;
    else if constexpr (KIND == KIND_THIN && NPT1 == 2)
        return thin_conv_pool_kernel<NRT1>;          // Cin; 3x3 stride 2 -> pooling 3x3 stride 2
    else if constexpr (KIND == KIND_THIN)
        return thin_conv_kernel<NRT1, K1, K2B>;      // Cin, K, pooling window
    else
        return block_kernel<KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1>;
}

static BlockKernel kernel_of(int variant)
{
    switch (variant) {
#define X(ID, KIND, MF1, K1, NRT1, NPT1, MF2, NRT2, NPT2, K2A, K2B, SC, PX1)                       \
    case ID:                                                                                       \
        return select_kernel<KIND, MF1, K1, NRT1, NPT1, (MF2 == 0 ? 32 : MF2), (NRT2 == 0 ? 1 : NRT2), \
                             (NPT2 == 0 ? 1 : NPT2), (K2A == 0 ? 1 : K2A), K2B, (SC != 0), PX1>();
        XL_VARIANT_LIST(X)
#undef X
    }
    return kernel_of_b3(variant);
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
    if (p.nblocks <= 0) return hipSuccess;
    int grid = (p.nblocks + 7) / 8 * 8;
    if (p.stream_wgs > 0) grid = std::min(grid, (p.stream_wgs + 7) / 8 * 8);     // resident workgroups walking the tiles
    return launch(k, dim3(grid), dim3(threads), lds_bytes, s, p);
}

// ----------------------------------------------------------------------------
// filter re-layout: [Cout][Cin][K][K] -> [K step][tap][row tile][lane] float4
//   MF = 32: lane l holds cout = rt*32 + l%32, cin = kg*8  + (l/32)*4 + j
//   MF = 16: lane l holds cout = rt*16 + l%16, cin = kg*16 + (l/16)*4 + j
// zero where cout or cin run past the real extent.
// ----------------------------------------------------------------------------
// pairs != 0 (mf = 32, one K step): channel c goes to lane half c % 2, slot c / 2.
__global__ void pack_filter_kernel(const float *__restrict__ w, const float *__restrict__ scale, f32x4 *__restrict__ wp,
                                   int cout, int cin, int k, int mf, int nkg, int nrt, int pairs)
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
        const int ci = pairs ? 2 * j + sub : kg * kc + sub * 4 + j;
        v[j] = (o < cout && ci < cin) ? w[((size_t)o * cin + ci) * taps + t] * (scale ? scale[o] : 1.f) : 0.f;
    }
    wp[idx] = v;
}

// split-bf16 form: [K step][tap][row tile][hi, lo][lane] of 8 bf16;
//   lane l holds cout = rt*mf + l%mf, cin = kg*kc + (l/mf)*8 + e, kc = 16 (mf = 32) or 32 (mf = 16);
//   hi = bf16(w), lo = bf16(w - hi), round to nearest.
__global__ void pack_filter_b3_kernel(const float *__restrict__ w, const float *__restrict__ scale, uint4 *__restrict__ wp,
                                      int cout, int cin, int k, int mf, int nkg, int nrt)
{
    const int taps = k * k;
    const long long total = (long long)nkg * taps * nrt * 128;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const int part = (int)((idx >> 6) & 1);
    long long r = idx >> 7;
    const int rt = (int)(r % nrt);
    r /= nrt;
    const int t = (int)(r % taps);
    const int kg = (int)(r / taps);
    const int o = rt * mf + lane % mf;
    const int sub = lane / mf;
    const int kc = mf == 32 ? 16 : 32;
    unsigned out[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float v[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ci = kg * kc + sub * 8 + 2 * e + h;
            v[h] = (o < cout && ci < cin) ? w[((size_t)o * cin + ci) * taps + t] * (scale ? scale[o] : 1.f) : 0.f;
        }
        unsigned hi, lo;
        split_bf16(v[0], v[1], hi, lo);
        out[e] = part ? lo : hi;
    }
    wp[idx] = uint4{out[0], out[1], out[2], out[3]};
}

hipError_t launch_pack_filter(const float *w, const float *scale, f32x4 *wp, int cout, int cin, int k, int mf, int nkg,
                              int nrt, hipStream_t s, int pairs, int pr)
{
    const long long total = (long long)nkg * k * k * nrt * (pr ? 128 : 64);
    const int threads = 256;
    const int grid = (int)((total + threads - 1) / threads);
    if (pr)
        return launch(pack_filter_b3_kernel, dim3(grid), dim3(threads), 0, s, w, scale, (uint4 *)wp, cout, cin, k, mf, nkg, nrt);
    return launch(pack_filter_kernel, dim3(grid), dim3(threads), 0, s, w, scale, wp, cout, cin, k, mf, nkg, nrt, pairs);
}

hipError_t launch_pack_thin(const float *w, const float *scale, const float *shift, float *wp, float *aff, int cout,
                            int taps, hipStream_t s)
{
    const int total = (cout + 15) / 16 * 16 * thin_row_floats(taps);
    return launch(pack_thin_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w, scale, shift, wp, aff, cout, taps);
}

// shift in accumulator order: [row tile][quad][lane] float4 (the scale goes into the filter)
__global__ void pack_affine_kernel(const float *__restrict__ shift, f32x4 *__restrict__ out, int cout, int mf, int nrt)
{
    const int nq = mf == 32 ? 4 : 1;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // over nrt * nq * 64
    if (idx >= nrt * nq * 64) return;
    const int lane = idx & 63, q = (idx >> 6) % nq, rt = (idx >> 6) / nq;
    const int sub = lane / mf;
    const int cb = rt * mf + (mf == 32 ? q * 8 + sub * 4 : sub * 4);
    f32x4 b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int co = cb + i;
        b[i] = (co < cout && shift) ? shift[co] : 0.f;
    }
    out[idx] = b;
}

hipError_t launch_pack_affine(const float *shift, f32x4 *out, int cout, int mf, int nrt, hipStream_t s)
{
    const int total = nrt * (mf == 32 ? 4 : 1) * 64;
    return launch(pack_affine_kernel, dim3((total + 255) / 256), dim3(256), 0, s, shift, out, cout, mf, nrt);
}

// ----------------------------------------------------------------------------
// element-wise layers of the unfused path
// ----------------------------------------------------------------------------
// one thread per output element; blockIdx.x = image * C + channel, blockIdx.y = block of pixels
// (32-bit index math only)
__global__ void maxpool_kernel(const float *__restrict__ x, float *__restrict__ y, int C, int H, int W, int Ho, int Wo,
                               int k, int stride, int pad, int Cy, int coff)
{
    const int idx = blockIdx.y * blockDim.x + threadIdx.x;
    if (idx >= Ho * Wo) return;
    const int oy = idx / Wo, ox = idx - oy * Wo;
    const int plane = blockIdx.x;
    const int n = plane / C, c = plane - n * C;
    const float *xc = x + (size_t)plane * H * W;
    const int y0 = oy * stride - pad, x0 = ox * stride - pad;
    float m = -FLT_MAX;
    for (int u = 0; u < k; ++u) {
        const int yy = y0 + u;
        if (yy < 0 || yy >= H) continue;
        for (int v = 0; v < k; ++v) {
            const int xx = x0 + v;
            if (xx < 0 || xx >= W) continue;
            m = fmaxf(m, xc[yy * W + xx]);
        }
    }
    y[((size_t)n * Cy + coff + c) * Ho * Wo + idx] = m;
}

// Planes that fit LDS: one workgroup per (image, channel) plane copies it into LDS with 16-byte
// loads (any 4-byte alignment), then every thread pools from LDS.
typedef float f32x4_unaligned __attribute__((ext_vector_type(4), aligned(4)));

__global__ void __launch_bounds__(256) maxpool_plane_kernel(const float *__restrict__ x, float *__restrict__ y, int C,
                                                            int H, int W, int Ho, int Wo, int k, int stride, int pad,
                                                            int Cy, int coff)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int plane = blockIdx.x;
    const int n = plane / C, c = plane - n * C;
    const int HW = H * W;
    const float *xc = x + (size_t)plane * HW;
    const int n4 = HW >> 2;
    for (int i = threadIdx.x; i < n4; i += blockDim.x) *(f32x4 *)(lds + i * 4) = *(const f32x4_unaligned *)(xc + i * 4);
    for (int i = (n4 << 2) + threadIdx.x; i < HW; i += blockDim.x) lds[i] = xc[i];
    __syncthreads();
    float *yc = y + ((size_t)n * Cy + coff + c) * Ho * Wo;
    for (int idx = threadIdx.x; idx < Ho * Wo; idx += blockDim.x) {
        const int oy = idx / Wo, ox = idx - oy * Wo;
        const int y0 = oy * stride - pad, x0 = ox * stride - pad;
        float m = -FLT_MAX;
        for (int u = 0; u < k; ++u) {
            const int yy = y0 + u;
            if (yy < 0 || yy >= H) continue;
            for (int v = 0; v < k; ++v) {
                const int xx = x0 + v;
                if (xx < 0 || xx >= W) continue;
                m = fmaxf(m, lds[yy * W + xx]);
            }
        }
        yc[idx] = m;
    }
}

hipError_t launch_maxpool(const float *x, float *y, int N, int C, int H, int W, int Ho, int Wo, int k, int stride,
                          int pad, int Cy, int coff, hipStream_t s)
{
    if ((long long)N * C * Ho * Wo == 0) return hipSuccess;
    const int threads = 256;
    const size_t plane_bytes = (size_t)H * W * 4;
    if (plane_bytes <= 64 * 1024) {
        return launch(maxpool_plane_kernel, dim3(N * C), dim3(threads), (plane_bytes + 15) / 16 * 16, s, x, y, C, H,
                           W, Ho, Wo, k, stride, pad, Cy, coff);
    }
    const int pix_blocks = (Ho * Wo + threads - 1) / threads;
    if (pix_blocks > 65535) return hipErrorInvalidValue;
    return launch(maxpool_kernel, dim3(N * C, pix_blocks), dim3(threads), 0, s, x, y, C, H, W, Ho, Wo, k, stride,
                       pad, Cy, coff);
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
    return launch(add_kernel, dim3((unsigned)((work + threads - 1) / threads)), dim3(threads), 0, s, a, b, y, count,
                       relu);
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
    return launch(gap_kernel, dim3((NC + wpb - 1) / wpb), dim3(threads), 0, s, x, y, NC, HW);
}

// ----------------------------------------------------------------------------
// Peak probes: what the device sustains on a plain copy and on register-only arithmetic loops
// ----------------------------------------------------------------------------
__global__ void __launch_bounds__(256) probe_copy_kernel(f32x4 *__restrict__ dst, const f32x4 *__restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

constexpr int PROBE_ITERS = 4096;

// 4 independent accumulator tiles per wave: the matrix pipe never waits for a result
__global__ void __launch_bounds__(512) probe_mfma_f32_kernel(float *out, float a0)
{
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) zero_acc(acc[i]);
    const float a = a0 + threadIdx.x, b = a0 * 0.5f;
    for (int it = 0; it < PROBE_ITERS; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ void __launch_bounds__(512) probe_mfma_bf16_kernel(float *out, float a0)
{
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) zero_acc(acc[i]);
    const f32x4 av = {a0, a0 + threadIdx.x, a0, a0}, bv = {a0, a0, a0 * 0.5f, a0};
    const bf16x8 a = __builtin_bit_cast(bf16x8, av), b = __builtin_bit_cast(bf16x8, bv);
    for (int it = 0; it < PROBE_ITERS; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 16 independent chains of multiply-adds per lane
__global__ void __launch_bounds__(512) probe_valu_kernel(float *out, float a0)
{
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = a0 + i + threadIdx.x;
    const float m = 1.0f + a0 * 1e-7f, c = a0 * 1e-3f;
    for (int it = 0; it < PROBE_ITERS; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = fmaf(acc[i], m, c);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

hipError_t launch_peak_probe(int what, void *dst, const void *src, size_t bytes, int num_cus, hipStream_t s, double *work)
{
    const int wgs = num_cus * 4, threads = 512;         // 2 MiB of sink: wgs * threads floats
    const double waves = (double)wgs * (threads / 64);
    switch (what) {
    case 0:
        *work = 2.0 * (double)(bytes / 16 * 16);
        return launch(probe_copy_kernel, dim3(num_cus * 8), dim3(256), 0, s, (f32x4 *)dst, (const f32x4 *)src, bytes / 16);
    case 1:
        *work = waves * PROBE_ITERS * 4 * (2.0 * 32 * 32 * 2);
        return launch(probe_mfma_f32_kernel, dim3(wgs), dim3(threads), 0, s, (float *)dst, 1.0f);
    case 2:
        *work = waves * PROBE_ITERS * 4 * (2.0 * 32 * 32 * 16);
        return launch(probe_mfma_bf16_kernel, dim3(wgs), dim3(threads), 0, s, (float *)dst, 1.0f);
    case 3:
        *work = waves * PROBE_ITERS * 16 * 64 * 2.0;
        return launch(probe_valu_kernel, dim3(wgs), dim3(threads), 0, s, (float *)dst, 1.0f);
    }
    return hipErrorInvalidValue;
}

// ----------------------------------------------------------------------------
// Depthwise convolution (groups == channels): tables and the per-layer kernel of the unfused path
// ----------------------------------------------------------------------------
// [C][1][K][K] -> [channel group][tap] float4, and scale / shift -> [channel group][2] float4
// (scale 1 / shift 0 where the pointer is null, zero filter and tables for channels past C).
__global__ void pack_depthwise_kernel(const float *__restrict__ w, const float *__restrict__ scale,
                                      const float *__restrict__ shift, f32x4 *__restrict__ wp, f32x4 *__restrict__ aff,
                                      int C, int taps)
{
    const int ncg = (C + 3) >> 2;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < ncg * taps) {
        const int g = idx / taps, t = idx - g * taps;
        f32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (g * 4 + j < C) ? w[(g * 4 + j) * taps + t] : 0.f;
        wp[idx] = v;
    }
    if (idx < ncg) {
        f32x4 a, b;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = idx * 4 + j;
            a[j] = c < C ? (scale ? scale[c] : 1.f) : 0.f;
            b[j] = c < C ? (shift ? shift[c] : 0.f) : 0.f;
        }
        aff[idx * 2] = a;
        aff[idx * 2 + 1] = b;
    }
}

hipError_t launch_pack_depthwise(const float *w, const float *scale, const float *shift, f32x4 *wp, f32x4 *aff, int C,
                                 int k, hipStream_t s)
{
    const int items = ((C + 3) / 4) * k * k;
    return launch(pack_depthwise_kernel, dim3((items + 255) / 256), dim3(256), 0, s, w, scale, shift, wp, aff, C,
                       k * k);
}

// one thread per output element; consecutive threads run along W
__global__ void depthwise_kernel(const float *__restrict__ x, float *__restrict__ y, const f32x4 *__restrict__ wp,
                                 const f32x4 *__restrict__ aff, int C, int H, int W, int Ho, int Wo, int k, int stride,
                                 int pad, int relu, int Cy, int coff, long long total)
{
    const long long idx = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int ox = (int)(idx % Wo);
    long long r = idx / Wo;
    const int oy = (int)(r % Ho);
    r /= Ho;
    const int c = (int)(r % C);
    const long long n = r / C;
    const float *xc = x + ((size_t)n * C + c) * H * W;
    const int g = c >> 2, j = c & 3;
    float a = 0.f;
    for (int u = 0; u < k; ++u) {
        const int iy = oy * stride - pad + u;
        if (iy < 0 || iy >= H) continue;
        for (int v = 0; v < k; ++v) {
            const int ix = ox * stride - pad + v;
            if (ix < 0 || ix >= W) continue;
            a = fmaf(xc[iy * W + ix], wp[g * k * k + u * k + v][j], a);
        }
    }
    float t = a * aff[g * 2][j] + aff[g * 2 + 1][j];
    if (relu) t = fmaxf(t, 0.f);
    y[(((size_t)n * Cy + coff + c) * Ho + oy) * Wo + ox] = t;
}

hipError_t launch_depthwise(const float *x, float *y, const f32x4 *wp, const f32x4 *aff, int N, int C, int H, int W,
                            int Ho, int Wo, int k, int stride, int pad, int relu, int Cy, int coff, hipStream_t s)
{
    const long long total = (long long)N * C * Ho * Wo;
    if (total == 0) return hipSuccess;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    return launch(depthwise_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x, y, wp, aff, C, H, W, Ho, Wo, k, stride,
                       pad, relu, Cy, coff, total);
}

#endif  // XL_TU_B3

}  // namespace xl

