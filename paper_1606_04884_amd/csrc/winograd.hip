// Winograd F(2x2,3x3) convolution on fp32 MFMA for gfx950: forward and
// backward-data of 3x3 stride-1 layers, fused into one kernel per call.
//
// Sec. 4.2 "Winograd" of the paper: minimal filtering cuts the multiplications
// of a 3x3 convolution by 2.25 while the bulk of the work remains matrix products;
// Sec. 4.2 "Neon": the fast implementations fuse the transforms into those products.  The paper
// prints no transform matrices; the standard ones for the points {0,1,-1,inf}
// are used:
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]     (input tile d, 4x4)
//   G   = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]          (filter g, 3x3)
//   A^T = [1 1 1 0; 0 1 -1 -1]                         (output, 2x2)
//   Y = A^T [ sum_c (G g G^T) .* (B^T d B) ] A
// The sum over c at each of the 16 positions is a GEMM  M[pos] = U[pos]^T V[pos]
// with U[pos] : [C x K] (filters), V[pos] : [C x tiles].
//
// One workgroup (4 waves) computes 64 filters x 64 tiles at all 16 positions: each
// wave keeps 16 accumulator tiles of 32x32 (256 accumulator registers), so the
// output transform needs no exchange: the 16 values of one (filter, tile) sit in
// the same lane and register index of the 16 accumulators.  Per 8-channel chunk
// the input patches are loaded from NCHW, transformed in registers and written
// to LDS as V; the pre-transformed filters U are copied to LDS; nothing
// transformed ever goes to HBM except U (16*C*K floats, written once per call).
// One wave per SIMD, so the whole latency hiding is the in-wave software
// pipeline: LDS operand prefetch one position pair ahead, LDS writes of chunk
// t+1 and global loads of chunk t+2 interleaved between the MFMAs of chunk t,
// LDS-only barrier hidden under the last position pair.

#include "conv_internal.h"

#include <mutex>

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// --------------------------------------------------------- filter transform
// U[pos][c'][k] (k contiguous, zero padded to Cpad x Kpad).  A filter larger than
// 3x3 is the sum of 3x3 sub-filters applied to shifted inputs: virtual channel
// c' = q * Cin + c carries sub-filter q = (a, b) of channel c, taps (3a + r, 3b + s),
// zero where the R x S filter ends (R = S = 3: one sub-filter, the filter itself).
// mode 0: forward, filters g = w[k][c].  mode 1: backward-data, the layer that
// maps dy to dx has filters g'[c][k][r][s] = w[k][c][R-1-r][S-1-s]; its "k" is c.
__global__ __launch_bounds__(256) void wino_filter_kernel(const float *__restrict__ w,
                                                          float *__restrict__ U, int K, int C,
                                                          int R, int S, int Cin, int Kout,
                                                          int Cpad, int Kpad, int mode)
{
    const int64_t total = (int64_t)Cpad * Kpad;
    const int nsw = (S + 2) / 3;
    const int RS = R * S;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int cv = (int)(i / Kpad), ko = (int)(i - (int64_t)cv * Kpad);
        const int q = cv / Cin, ci = cv - q * Cin;
        const int r0 = 3 * (q / nsw), s0 = 3 * (q - (q / nsw) * nsw);
        float g[3][3];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) g[r][s] = 0.f;
        if (ko < Kout) {
            const float *p = mode == 0 ? w + ((int64_t)ko * C + ci) * RS : w + ((int64_t)ci * C + ko) * RS;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const int rr = r0 + r, ss = s0 + s;
                    if (rr < R && ss < S) g[r][s] = mode == 0 ? p[rr * S + ss] : p[(R - 1 - rr) * S + (S - 1 - ss)];
                }
        }
        float t[4][3];
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            t[0][s] = g[0][s];
            t[1][s] = 0.5f * (g[0][s] + g[1][s] + g[2][s]);
            t[2][s] = 0.5f * (g[0][s] - g[1][s] + g[2][s]);
            t[3][s] = g[2][s];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float u0 = t[r][0];
            const float u1 = 0.5f * (t[r][0] + t[r][1] + t[r][2]);
            const float u2 = 0.5f * (t[r][0] - t[r][1] + t[r][2]);
            const float u3 = t[r][2];
            U[(int64_t)(4 * r + 0) * total + i] = u0;
            U[(int64_t)(4 * r + 1) * total + i] = u1;
            U[(int64_t)(4 * r + 2) * total + i] = u2;
            U[(int64_t)(4 * r + 3) * total + i] = u3;
        }
    }
}

// The same transform writing the paired layout U[pos][c/8][c%2][k][(c%8)/2]: a
// thread owns the four channels c = 8*chunk + half + 2*ks (ks = 0..3) of one filter
// and stores each position as one 16-byte vector.
__global__ __launch_bounds__(256) void wino_filter_paired_kernel(const float *__restrict__ w,
                                                                 float *__restrict__ U, int C,
                                                                 int Cin, int Kout, int Cpad, int Kpad,
                                                                 int mode)
{
    const int64_t total = (int64_t)Cpad * Kpad;           // floats per position
    const int64_t nvec = total / 4;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec;
         v += (int64_t)gridDim.x * blockDim.x) {
        const int ko = (int)(v % Kpad);
        const int ch = (int)(v / Kpad);                   // chunk * 2 + half
        floatx4 u[16];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int ci = (ch >> 1) * 8 + (ch & 1) + 2 * ks;
            float g[3][3];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s2 = 0; s2 < 3; ++s2) g[r][s2] = 0.f;
            if (ci < Cin && ko < Kout) {
                if (mode == 0) {
                    const float *p = w + ((int64_t)ko * C + ci) * 9;
#pragma unroll
                    for (int r = 0; r < 3; ++r)
#pragma unroll
                        for (int s2 = 0; s2 < 3; ++s2) g[r][s2] = p[r * 3 + s2];
                } else {
                    const float *p = w + ((int64_t)ci * C + ko) * 9;
#pragma unroll
                    for (int r = 0; r < 3; ++r)
#pragma unroll
                        for (int s2 = 0; s2 < 3; ++s2) g[r][s2] = p[(2 - r) * 3 + (2 - s2)];
                }
            }
            float t[4][3];
#pragma unroll
            for (int s2 = 0; s2 < 3; ++s2) {
                t[0][s2] = g[0][s2];
                t[1][s2] = 0.5f * (g[0][s2] + g[1][s2] + g[2][s2]);
                t[2][s2] = 0.5f * (g[0][s2] - g[1][s2] + g[2][s2]);
                t[3][s2] = g[2][s2];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u[4 * r + 0][ks] = t[r][0];
                u[4 * r + 1][ks] = 0.5f * (t[r][0] + t[r][1] + t[r][2]);
                u[4 * r + 2][ks] = 0.5f * (t[r][0] - t[r][1] + t[r][2]);
                u[4 * r + 3][ks] = t[r][2];
            }
        }
#pragma unroll
        for (int pos = 0; pos < 16; ++pos)
            *reinterpret_cast<floatx4 *>(U + (int64_t)pos * total + v * 4) = u[pos];
    }
}

hipError_t launch_wino_filter(const float *w, float *U, int K, int C, int R, int S, int Cin, int Kout,
                              int Cpad, int Kpad, int mode, int paired, hipStream_t s)
{
    if (paired) {       // 3x3 only
        int64_t blocks = ((int64_t)Cpad * Kpad / 4 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(wino_filter_paired_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, U, C,
                           Cin, Kout, Cpad, Kpad, mode);
        return hipGetLastError();
    }
    int64_t blocks = ((int64_t)Cpad * Kpad + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(wino_filter_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, U, K, C, R, S,
                       Cin, Kout, Cpad, Kpad, mode);
    return hipGetLastError();
}

// ------------------------------------------------------------- fused kernel
__device__ __forceinline__ void lds_barrier_wg()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ int xcd_remap_wino(int id, int nb)
{
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = id & 7, local = id >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}


constexpr int kWinoKB = 64, kWinoTB = 64, kWinoCB = 8;
constexpr int kWinoLdsBytes = 2 * 16 * kWinoCB * (kWinoKB + kWinoTB) * (int)sizeof(float);

// Range of units of one persistent workgroup and the lane's place in the
// accumulator layout, for the tile epilogue shared by the fused kernels.
struct WinoTileCtx {
    int ub, ue, lb, nchunks;
    int wm0, wn0, l32, lhi;
};

// Output transform of the finished (or cut) tile in registers; accumulator
// element v of lane L: filter row 8*(v/4) + 4*(L/32) + v%4, tile column L%32.
// Tiles whose first output column lies outside the map (phantom tiles of a tile
// grid taken wider than the map) are computed but not stored.
template <bool ZERO>
__device__ __forceinline__ void wino_finish_tile(const WinoArgs &a, floatx16 (&acc)[16], int tile_id,
                                                 int first_unit, const WinoTileCtx &cx)
{
    constexpr int KB = kWinoKB, TB = kWinoTB;
    const int ub = cx.ub, ue = cx.ue, lb = cx.lb, nchunks = cx.nchunks;
    const int wm0 = cx.wm0, wn0 = cx.wn0, l32 = cx.l32, lhi = cx.lhi;

    const int kt = tile_id / a.tiles_t, tt = tile_id - kt * a.tiles_t;
    const bool head = first_unit < ub, tail = first_unit + nchunks > ue;
    float *slot = a.partial + ((int64_t)lb * 2 + (head ? 0 : 1)) * (KB * TB * 4);
    const int tile = tt * TB + wn0 + l32;
    const int tl = tile < a.T ? tile : 0;
    const int n = tl / (a.TH * a.TW), rem = tl - n * (a.TH * a.TW);
    const int th = rem / a.TW, tw = rem - th * a.TW;
    const int oh = 2 * th, ow = 2 * tw;
    const bool tv = tile < a.T && ow < a.Wout;
    const bool row1 = oh + 1 < a.Hout, col1 = ow + 1 < a.Wout;
    const int HWo = a.Hout * a.Wout;
    float *obase = a.out + (int64_t)n * a.Kout * HWo + (int64_t)oh * a.Wout + ow;
    // 2x2 outputs of accumulator element v (without bias)
    auto out_xform = [&](int v, float &y00, float &y01, float &y10, float &y11) {
        float s0[4], s1[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m0 = acc[0 + j][v], m1 = acc[4 + j][v], m2 = acc[8 + j][v], m3 = acc[12 + j][v];
            s0[j] = m0 + m1 + m2;
            s1[j] = m1 - m2 - m3;
        }
        y00 = s0[0] + s0[1] + s0[2]; y01 = s0[1] - s0[2] - s0[3];
        y10 = s1[0] + s1[1] + s1[2]; y11 = s1[1] - s1[2] - s1[3];
    };
    // (the 16 rounds are kept apart by scheduling fences: scheduled together they
    // would need all 256 accumulator values in ordinary registers at once)
    if (head || tail) {
        float *sp = slot + ((wm0 + 4 * lhi) * TB + wn0 + l32) * 4;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            __builtin_amdgcn_sched_barrier(0);
            float y00, y01, y10, y11;
            out_xform(v, y00, y01, y10, y11);
            const floatx4 o4 = {y00, y01, y10, y11};
            *reinterpret_cast<floatx4 *>(sp + ((8 * (v >> 2) + (v & 3)) * TB) * 4) = o4;
        }
    } else if (tv) {
        const int kbase = kt * KB + wm0 + 4 * lhi;
        float *ob = obase + (int64_t)kbase * HWo;
        const float *bp = a.bias ? a.bias + kbase : nullptr;
        if (a.pool) {
            // 2x2 / stride-2 max pooling of the rectified output: a tile's 2x2 block is one
            // pooled pixel (Hout and Wout are even)
            const int HWp = HWo >> 2;
            float *opl = a.out + ((int64_t)n * a.Kout + kbase) * HWp + th * (a.Wout >> 1) + tw;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                __builtin_amdgcn_sched_barrier(0);
                const int kr = 8 * (v >> 2) + (v & 3);
                if (kbase + kr < a.Kout) {
                    float y00, y01, y10, y11;
                    out_xform(v, y00, y01, y10, y11);
                    const float bz = bp ? bp[kr] : 0.f;
                    opl[(int64_t)kr * HWp] = fmaxf(fmaxf(fmaxf(y00, y01), fmaxf(y10, y11)) + bz, 0.f);
                }
            }
        } else if (a.vec2) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                __builtin_amdgcn_sched_barrier(0);
                const int kr = 8 * (v >> 2) + (v & 3);
                if (kbase + kr < a.Kout) {
                    float y00, y01, y10, y11;
                    out_xform(v, y00, y01, y10, y11);
                    const float bz = bp ? bp[kr] : 0.f;
                    float *o = ob + (int64_t)kr * HWo;
                    y00 += bz; y01 += bz; y10 += bz; y11 += bz;
                    if (a.relu) { y00 = fmaxf(y00, 0.f); y01 = fmaxf(y01, 0.f); y10 = fmaxf(y10, 0.f); y11 = fmaxf(y11, 0.f); }
                    *reinterpret_cast<float2 *>(o) = make_float2(y00, y01);
                    if (row1) *reinterpret_cast<float2 *>(o + a.Wout) = make_float2(y10, y11);
                }
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                __builtin_amdgcn_sched_barrier(0);
                const int kr = 8 * (v >> 2) + (v & 3);
                if (kbase + kr < a.Kout) {
                    float y00, y01, y10, y11;
                    out_xform(v, y00, y01, y10, y11);
                    const float bz = bp ? bp[kr] : 0.f;
                    float *o = ob + (int64_t)kr * HWo;
                    y00 += bz; y01 += bz; y10 += bz; y11 += bz;
                    if (a.relu) { y00 = fmaxf(y00, 0.f); y01 = fmaxf(y01, 0.f); y10 = fmaxf(y10, 0.f); y11 = fmaxf(y11, 0.f); }
                    o[0] = y00;
                    if (col1) o[1] = y01;
                    if (row1) {
                        o[a.Wout] = y10;
                        if (col1) o[a.Wout + 1] = y11;
                    }
                }
            }
        }
    }
    if (ZERO) {
#pragma unroll
        for (int p = 0; p < 16; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;
    }
}

// Work decomposition ("stream-K"): a unit is one 8-channel chunk of one output
// tile (64 filters x 64 tiles); units are numbered chunk-fastest, then tile block,
// then filter tile.  The grid is persistent: workgroup b processes the contiguous
// unit range [b*U/G, (b+1)*U/G), so every compute unit gets the same amount of
// MFMA work whatever the layer's tile count, and the software pipeline simply
// runs on across tile boundaries (the loads of the next tile's first chunks are
// in flight while the previous tile's epilogue runs).  An output tile that lies
// entirely inside a range is finished there (output transform, bias, store); a
// tile cut by a range boundary is written, output-transformed but without bias,
// to the range's head or tail slot in the workspace, and wino_fixup_kernel adds
// the two halves in a fixed order.  G <= number of tiles, so a tile is cut at
// most once.
//
// VEC: patch rows are fetched as dword + 8-byte + dword; needs pad_w <= 1 and an
// even width so that the middle two columns are always inside the image.
template <bool VEC>
__global__ __launch_bounds__(256, 1) void wino_fused_kernel(WinoArgs a)
{
    constexpr int KB = kWinoKB, TB = kWinoTB, CB = kWinoCB;
    extern __shared__ float lds[];
    // Us[buf][pos][c][k], Vs[buf][pos][c][tile]
    float *const Us = lds;
    float *const Vs = lds + 2 * 16 * CB * KB;
    auto us_at = [&](int buf, int pos, int c, int k) -> float & { return Us[((buf * 16 + pos) * CB + c) * KB + k]; };
    auto vs_at = [&](int buf, int pos, int c, int t) -> float & { return Vs[((buf * 16 + pos) * CB + c) * TB + t]; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;

    // XCD-contiguous ranges: an XCD then works on few filter tiles at a time and
    // keeps their slices of U in its L2
    const int G = gridDim.x;
    const int lb = xcd_remap_wino(blockIdx.x, G);
    const int ub = (int)((int64_t)lb * a.units_total / G);
    const int ue = (int)((int64_t)(lb + 1) * a.units_total / G);
    const int nunits = ue - ub;
    if (nunits <= 0) return;
    const int nchunks = a.nchunks;

    // Patch elements are fetched with buffer loads: the per-thread byte offset of
    // each element (inside channel 0 of its image) is fixed per tile block, the
    // channel advances through the scalar offset, and elements outside the image
    // carry an offset beyond the buffer, for which the hardware range check (done
    // per dword) returns 0: zero padding costs no instruction.
    const int HW = a.Hin * a.Win;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, a.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ursrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.U, 0, a.u_bytes, 0x00020000);
    uint32_t eoff[16];      // byte offset of patch element 4*i+j inside channel 0 (or 2^31)
    // (tt: tile block; q: sub-filter group, whose input is shifted by (sub_dh, sub_dw))
    const int nch_c = nchunks / a.nsub;               // chunks per sub-filter group
    auto set_tile_block = [&](int tt, int q) {
        const int tile = tt * TB + lane;
        const bool tv = tile < a.T;
        const int tl = tv ? tile : 0;
        const int n = tl / (a.TH * a.TW), rem = tl - n * (a.TH * a.TW);
        const int th = rem / a.TW, tw = rem - th * a.TW;
        const int dh = q == 0 ? a.sub_dh[0] : q == 1 ? a.sub_dh[1] : q == 2 ? a.sub_dh[2] : a.sub_dh[3];
        const int dw = q == 0 ? a.sub_dw[0] : q == 1 ? a.sub_dw[1] : q == 2 ? a.sub_dw[2] : a.sub_dw[3];
        const int ih0 = 2 * th - a.pad_h + dh, iw0 = 2 * tw - a.pad_w + dw;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (VEC && j == 2) continue;        // fetched together with column 1
                const bool ok = tv && (unsigned)(ih0 + i) < (unsigned)a.Hin &&
                                (unsigned)(iw0 + j) < (unsigned)a.Win;
                const int idx = n * a.Cin * HW + (ih0 + i) * a.Win + (iw0 + j);
                eoff[4 * i + j] = ok ? (uint32_t)idx * 4u : 0x80000000u;
            }
    };
    // wave w transforms channels w and w+4 of every chunk
    const int x_chunk = CB * HW * 4;                  // bytes per chunk of channels
    const int xs0 = wave * HW * 4, xs1 = xs0 + 4 * HW * 4;

    // U tile copy: 8 float4 per thread per chunk; vector v = tid + 256*i ->
    // pos = 2*i + tid/128, row = (tid%128)/16, column quad = tid%16
    const int u_row = (tid & 127) >> 4, u_c4 = tid & 15, u_p0 = tid >> 7;
    // (vector i differs from vector 0 only by a uniform stride: it goes into the
    // scalar offset, leaving a single per-thread offset register)
    const uint32_t uoff0 = (uint32_t)((((int64_t)u_p0 * a.Cpad + u_row) * a.Kpad + u_c4 * 4) * 4);
    const int u_vec_stride = 2 * a.Cpad * a.Kpad * 4;
    const int u_chunk = CB * a.Kpad * 4;

    float xr[2][16];
    floatx4 ur[8];
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    constexpr int XLOADS = VEC ? 12 : 16;
    // load number l of an item.  VEC: row l/3: column 0, columns 1-2, column 3;
    // otherwise the 16 elements in column-major order (the order of consumption)
    auto load_x = [&](int it, int l, int chunk) {
        const int so = (chunk % nch_c) * x_chunk + (it ? xs1 : xs0);
        if (VEC) {
            const int i = l / 3, part = l - 3 * i;
            if (part == 1) {
                // (cast the whole result vector, then index the cast value)
                const floatx2 v = __builtin_bit_cast(
                    floatx2, __builtin_amdgcn_raw_buffer_load_b64(xrsrc, eoff[4 * i + 1], so, 0));
                xr[it][4 * i + 1] = v[0];
                xr[it][4 * i + 2] = v[1];
            } else {
                const int e = 4 * i + (part == 0 ? 0 : 3);
                xr[it][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, eoff[e], so, 0));
            }
        } else {
            const int e = 4 * (l & 3) + (l >> 2);
            xr[it][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, eoff[e], so, 0));
        }
    };
    auto load_u = [&](int i, int kt, int chunk) {
        ur[i] = __builtin_bit_cast(
            floatx4, __builtin_amdgcn_raw_buffer_load_b128(ursrc, uoff0, chunk * u_chunk + kt * (KB * 4) + i * u_vec_stride, 0));
    };

    // input transform of item `it`, in two stages of four pieces each
    float tr[2][16];
    auto xform_col = [&](int it, int j) {     // stage 1 on patch column j: t = B^T d
        const float d0 = xr[it][0 + j], d1 = xr[it][4 + j], d2 = xr[it][8 + j], d3 = xr[it][12 + j];
        tr[it][0 + j] = d0 - d2;
        tr[it][4 + j] = d1 + d2;
        tr[it][8 + j] = d2 - d1;
        tr[it][12 + j] = d1 - d3;
    };
    auto xform_row_store = [&](int buf, int it, int i) {   // stage 2 on row i: V = t B, to LDS
        const float t0 = tr[it][4 * i + 0], t1 = tr[it][4 * i + 1], t2 = tr[it][4 * i + 2], t3 = tr[it][4 * i + 3];
        const int c = wave + 4 * it;
        vs_at(buf, 4 * i + 0, c, lane) = t0 - t2;
        vs_at(buf, 4 * i + 1, c, lane) = t1 + t2;
        vs_at(buf, 4 * i + 2, c, lane) = t2 - t1;
        vs_at(buf, 4 * i + 3, c, lane) = t1 - t3;
    };
    auto store_u = [&](int buf, int i) {
        *reinterpret_cast<floatx4 *>(&us_at(buf, 2 * i + u_p0, u_row, u_c4 * 4)) = ur[i];
    };

    floatx16 acc[16];
#pragma unroll
    for (int p = 0; p < 16; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;

    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    float ao[2][2][4], bo[2][2][4];     // [register set][position of the pair][k-step]
    auto read_pair = [&](int buf, int pair, int set) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                ao[set][u][ks] = us_at(buf, 2 * pair + u, 2 * ks + lhi, wm0 + l32);
                bo[set][u][ks] = vs_at(buf, 2 * pair + u, 2 * ks + lhi, wn0 + l32);
            }
    };

    const WinoTileCtx cx = {ub, ue, lb, nchunks, wm0, wn0, l32, lhi};
    auto finish_tile = [&](int tile_id, int first_unit) { wino_finish_tile<true>(a, acc, tile_id, first_unit, cx); };

    // cursors (unit -> tile, chunk) of the three pipeline stages; units past the
    // end of the range are clamped to the last one (harmless reloads)
    const int ulast = ue - 1;
    auto tile_of = [&](int u) { return u / nchunks; };
    int c_tile = tile_of(ub), c_chunk = ub - c_tile * nchunks;          // compute: unit i
    int u_tile = c_tile, u_chunk_i = c_chunk;                            // filter loads: unit i+1
    int x_tile = c_tile, x_chunk_i = c_chunk;                            // patch loads: unit i+2
    auto advance = [&](int &tile, int &chunk, int &unit) {
        if (unit < ulast) {
            ++unit;
            if (++chunk == nchunks) { chunk = 0; ++tile; }
        }
    };
    int u_unit = ub, x_unit = ub;

    // ---- prologue: unit 0 into LDS buffer 0, patch loads of unit 1 ----
    // (the patch offsets depend on the tile block and on the sub-filter group)
    auto x_key = [&]() { return x_tile * a.nsub + x_chunk_i / nch_c; };
    auto set_x_block = [&]() { set_tile_block(x_tile % a.tiles_t, x_chunk_i / nch_c); };
    set_x_block();
#pragma unroll
    for (int it = 0; it < 2; ++it)
#pragma unroll
        for (int l = 0; l < XLOADS; ++l) load_x(it, l, x_chunk_i);
#pragma unroll
    for (int i = 0; i < 8; ++i) load_u(i, u_tile / a.tiles_t, u_chunk_i);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) xform_col(it, j);
#pragma unroll
        for (int i = 0; i < 4; ++i) xform_row_store(0, it, i);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) store_u(0, i);
    {
        const int before = x_key();
        advance(x_tile, x_chunk_i, x_unit);
        if (x_key() != before) set_x_block();
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int l = 0; l < XLOADS; ++l) load_x(it, l, x_chunk_i);
        advance(u_tile, u_chunk_i, u_unit);
    }
    lds_barrier_wg();
    read_pair(0, 0, 0);

    // 64 MFMA slots per unit i:
    //   slots  0..15 : input transform + LDS writes of unit i+1 (registers loaded
    //                  during unit i-1); slots 0..7 also issue the filter-tile
    //                  loads of unit i+1
    //   slots 16..47 : the patch loads of unit i+2
    //   slots 48..55 : filter tile of unit i+1 to LDS
    //   slot  56     : LDS-only barrier, then the first operands of unit i+1
    // Outer loop: one segment per output tile touched by the range; the inner loop
    // is the pipelined chunk loop, in which the accumulators are only ever used by
    // MFMAs (they stay in the accumulator register file); the output transform
    // runs between segments while the next tile's loads are already in flight.
    int first_unit = ub - c_chunk;          // first unit of the compute tile
    int i = 0;
    while (i < nunits) {
        int seg_end = i + (nchunks - c_chunk);
        if (seg_end > nunits) seg_end = nunits;
        for (; i < seg_end; ++i) {
            const int buf = i & 1;
            const int ukt = u_tile / a.tiles_t;
            {
                const int before = x_key();
                advance(x_tile, x_chunk_i, x_unit);
                // the patch registers still hold unit i+1 (transformed in slots 0..15);
                // the offsets are only used from slot 16 on
                if (x_key() != before) set_x_block();
            }
    #pragma unroll
            for (int pair = 0; pair < 8; ++pair) {
                const int cur = pair & 1, nxt = cur ^ 1;
                if (pair + 1 < 8) {
                    read_pair(buf, pair + 1, nxt);
                } else {
                    lds_barrier_wg();
                    read_pair(buf ^ 1, 0, nxt);
                }
    #pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int s = pair * 8 + q;      // MFMA slot 0..63 of this unit
                    if (s < 16) {
                        const int it = s >> 3, piece = s & 7;
                        if (piece < 4) xform_col(it, piece); else xform_row_store(buf ^ 1, it, piece - 4);
                        if (s < 8) load_u(s, ukt, u_chunk_i);
                    } else if (s < 48) {
                        const int l = s - 16;        // 32 slots for 2 * XLOADS loads
    #pragma unroll
                        for (int m = 0; m < 2 * XLOADS; ++m)
                            if (m * 32 / (2 * XLOADS) == l) load_x(m / XLOADS, m % XLOADS, x_chunk_i);
                    } else if (s < 56) {
                        store_u(buf ^ 1, s - 48);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    const int u = q & 1, ks = q >> 1;
                    acc[2 * pair + u] = __builtin_amdgcn_mfma_f32_32x32x2f32(ao[cur][u][ks], bo[cur][u][ks],
                                                                              acc[2 * pair + u], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            advance(u_tile, u_chunk_i, u_unit);
        }
        finish_tile(c_tile, first_unit);
        first_unit += nchunks;
        ++c_tile;
        c_chunk = 0;
    }
}

// ---------------------------------------------------------------------------
// Tile-pair kernel, for pad_w = 1, an even input width and an even number of tiles
// per row.
//
// Same decomposition (stream-K over 64 filters x 64 tiles x 16 positions) and the
// same result as wino_fused_kernel; what differs is how a chunk is staged, built
// on measurements on this chip: (1) fp32 MFMAs and other vector instructions do
// not overlap, a wave issues in order, and every switch between a run of MFMAs and
// other instructions costs a pipeline drain (~11 cycles): the MFMAs are issued in
// runs of 8 with all side work in the gaps; (2) a vector-memory instruction holds
// its wave for ~25 cycles when a few other instructions separate it from the next
// one and ~55 when loads are back to back: few, wide loads, spread between the
// other pieces; (3) LDS traffic costs the wave time in proportion to its bytes;
// (4) the side work of a wave can overlap the MFMAs of ANOTHER wave on its SIMD.
//   * A thread owns one channel of the chunk and a PAIR of horizontally adjacent
//     tiles: the two 4x4 patches are a 4 x 6 block, fetched per row as dword +
//     16 bytes + dword; the column half of B^T d B is shared by the two patches.
//     The tile grid has an even row width (the host picks this kernel only then),
//     so a pair never straddles two tile rows and the 16 bytes never leave the
//     image row.
//   * The V planes in LDS are [buf][pos][half][64 tiles][4]: the four channels a
//     lane needs for the four reduction steps of a chunk are 16 contiguous
//     bytes, one read per position; adjacent columns swap in the second
//     half-plane so that the stores of a half-wave (4 pairs x 8 channels) fall in
//     32 different banks.  The two buffers are 32 KB apart: switching is one XOR
//     per base register.
//   * The transformed filters do not go through LDS at all: the filter transform
//     writes U as [pos][chunk][half][filter][4], so the MFMA A operand of a lane
//     for one position of a chunk is 16 contiguous bytes of U, loaded straight
//     into the registers the MFMAs read (from L2).  The registers of a position
//     pair are reloaded for the next unit in the gap after their last MFMA.
//   * Eight waves, two per SIMD (point 4).  The 512 registers of a lane are split
//     between the two: a wave keeps 8 of the 16 positions of one 32x32 sub-tile
//     (128 accumulator registers).  Wave w: sub-tile sub = w % 4, position half
//     PH = w / 4; waves w and w + 4 share a SIMD.  Everything is split by PH:
//       - transform: a thread handles (tile pair, channel, PH): the 8 positions of
//         half PH are rows 2*PH, 2*PH+1 of B^T d B, which need only three of the
//         four patch rows (PH..PH+2): 9 loads, 12 + 16 adds, 8 paired LDS stores
//         per chunk;
//       - MFMA: positions 8*PH .. 8*PH+7 of the sub-tile, 4 runs of 8; B operands
//         from the V planes of half PH, which only the four waves of the same PH
//         write and read;
//       - epilogue: Y = A^T M A is a sum over the rows of M, so each wave reduces
//         its two rows to a partial 2x2 output per accumulator element; the
//         partials of the elements the partner finishes go through LDS (one
//         16-byte vector per element), a barrier, and each wave adds, applies the
//         bias and stores half of the elements.
// V planes (two buffers) + the exchange area of the epilogue
constexpr int kWinoPairLdsBytes = 2 * 16 * kWinoCB * kWinoTB * (int)sizeof(float) + 4 * 2 * 8 * 64 * 16;

// RAGGED: the channel count is not a multiple of the 8-channel chunk (first layers): the
// missing channels of the last chunk are fetched with offsets outside the buffer (zeros;
// their rows of U are zero too).
template <int PH, bool RAGGED>
__device__ __forceinline__ void wino_pair_body(const WinoArgs &a, float *lds)
{
    constexpr int KB = kWinoKB, TB = kWinoTB, CB = kWinoCB;
    constexpr int NX = 9;
    constexpr int PLANE = 512;                // floats per (buf, pos): 2 halves x 64 x 4
    constexpr int BUFSZ = 16 * PLANE;         // floats per buffer (32 KB)
    floatx4 *const lds4 = reinterpret_cast<floatx4 *>(lds);
    floatx4 *const xchg = lds4 + 2 * BUFSZ / 4;          // [sub][writer PH][8 elements][64 lanes]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int sub = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);
    const int l32 = lane & 31, lhi = lane >> 5;

    const int G = gridDim.x;
    const int lb = xcd_remap_wino(blockIdx.x, G);
    const int ub = (int)((int64_t)lb * a.units_total / G);
    const int ue = (int)((int64_t)(lb + 1) * a.units_total / G);
    const int nunits = ue - ub;
    if (nunits <= 0) return;
    const int nchunks = a.nchunks;

    const int pr = sub * 8 + (lhi << 2) + (lane & 3);     // tile pair of the block
    const int ch = (lane >> 2) & 7;                        // channel of the chunk
    const int HW = a.Hin * a.Win;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, a.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ursrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.U, 0, a.u_bytes, 0x00020000);
    // patch rows PH .. PH+2: byte offsets of the row pieces inside chunk 0, or 2^31
    uint32_t xo[3][3];
    auto set_tile_block = [&](int tt) {
        const int tile = tt * TB + 2 * pr;
        const bool tv = tile < a.T;
        const int tl = tv ? tile : 0;
        const int n = tl / (a.TH * a.TW), rem = tl - n * (a.TH * a.TW);
        const int th = rem / a.TW, tw = rem - th * a.TW;       // tw even
        const int ih0 = 2 * th - a.pad_h + PH, col0 = 2 * tw;
        const int base = (n * a.Cin + ch) * HW + ih0 * a.Win + col0;
        const bool lok = tw > 0, rgt = col0 + 4 < a.Win;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const bool rok = tv && (unsigned)(ih0 + i) < (unsigned)a.Hin;
            const uint32_t m = (uint32_t)(base + i * a.Win) * 4u;
            xo[i][0] = (rok && lok) ? m - 4u : 0x80000000u;
            xo[i][1] = rok ? m : 0x80000000u;
            xo[i][2] = (rok && rgt) ? m + 16u : 0x80000000u;
        }
    };
    const int x_chunk = CB * HW * 4;

    const int wm0 = (sub >> 1) * 32, wn0 = (sub & 1) * 32;
    const int u_plane = a.Kpad * 16;
    const int u_pos_stride = nchunks * 2 * u_plane;
    const int u_chunk = 2 * u_plane;
    const uint32_t aoff0 = (uint32_t)lhi * (uint32_t)u_plane + (uint32_t)(wm0 + l32) * 16u;
    const int a_pos0 = 8 * PH * u_pos_stride;

    float xr[3][6];
    floatx4 ar[8];
    // this lane's channel does not exist in the last chunk (RAGGED only)
    const uint32_t chbad = (RAGGED && (nchunks - 1) * CB + ch >= a.Cin) ? 0x80000000u : 0u;
    // x load l: part = l / 3 (left dword, 16 bytes, right dword), row = l % 3
    auto load_x = [&](int l, int chunk) {
        const int part = l / 3, i = l - 3 * part;
        const int so = chunk * x_chunk;
        const uint32_t bad = RAGGED ? (chbad & (chunk == nchunks - 1 ? 0xffffffffu : 0u)) : 0u;
        if (part == 0) {
            xr[i][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, xo[i][0] | bad, so, 0));
        } else if (part == 2) {
            xr[i][5] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, xo[i][2] | bad, so, 0));
        } else {
            const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, xo[i][1] | bad, so, 0));
            xr[i][1] = m[0]; xr[i][2] = m[1]; xr[i][3] = m[2]; xr[i][4] = m[3];
        }
    };
    auto load_a = [&](int p, int kt, int chunk) {
        ar[p] = __builtin_bit_cast(
            floatx4, __builtin_amdgcn_raw_buffer_load_b128(ursrc, aoff0, a_pos0 + chunk * u_chunk + kt * (KB * 16) + p * u_pos_stride, 0));
    };

    uint32_t wrV = 8 * PH * PLANE + (ch & 1) * 256 + (2 * pr + (ch & 1)) * 4 + (ch >> 1);
    uint32_t rdB = 8 * PH * PLANE + lhi * 256 + ((wn0 + l32) ^ lhi) * 4;
    auto flip = [&]() { wrV ^= BUFSZ; rdB ^= BUFSZ; };

    // rows 2*PH, 2*PH+1 of t = B^T d on column j of the pair (xr rows are patch rows PH..PH+2)
    float tc[2][6];
    auto xform_col = [&](int j) {
        const float e0 = xr[0][j], e1 = xr[1][j], e2 = xr[2][j];
        if (PH == 0) { tc[0][j] = e0 - e2; tc[1][j] = e1 + e2; }       // d0-d2, d1+d2
        else         { tc[0][j] = e1 - e0; tc[1][j] = e0 - e2; }       // d2-d1, d1-d3
    };
    auto xform_row_store = [&](int i, int h) {
        const float t0 = tc[i][2 * h + 0], t1 = tc[i][2 * h + 1], t2 = tc[i][2 * h + 2], t3 = tc[i][2 * h + 3];
        float *o = lds + (h ? wrV ^ 4u : wrV) + 4 * i * PLANE;
        o[0 * PLANE] = t0 - t2;
        o[1 * PLANE] = t1 + t2;
        o[2 * PLANE] = t2 - t1;
        o[3 * PLANE] = t1 - t3;
    };

    floatx16 acc[8];
#pragma unroll
    for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;

    floatx4 bo[2][2];
    auto read_b = [&](int pos, int set, int u) { bo[set][u] = lds4[(rdB >> 2) + pos * (PLANE / 4)]; };

    const int ulast = ue - 1;
    int c_tile = ub / nchunks, c_chunk = ub - c_tile * nchunks;
    int u_tile = c_tile, u_chunk_i = c_chunk;
    int x_tile = c_tile, x_chunk_i = c_chunk;
    auto advance = [&](int &tile, int &chunk, int &unit) {
        if (unit < ulast) {
            ++unit;
            if (++chunk == nchunks) { chunk = 0; ++tile; }
        }
    };
    int u_unit = ub, x_unit = ub;

    // ---- prologue ----
    set_tile_block(x_tile % a.tiles_t);
#pragma unroll
    for (int l = 0; l < NX; ++l) load_x(l, x_chunk_i);
#pragma unroll
    for (int p = 0; p < 8; ++p) load_a(p, u_tile / a.tiles_t, u_chunk_i);
#pragma unroll
    for (int j = 0; j < 6; ++j) xform_col(j);
#pragma unroll
    for (int q = 0; q < 4; ++q) xform_row_store(q >> 1, q & 1);
    {
        const int before = x_tile;
        advance(x_tile, x_chunk_i, x_unit);
        if (x_tile != before) set_tile_block(x_tile % a.tiles_t);
#pragma unroll
        for (int l = 0; l < NX; ++l) load_x(l, x_chunk_i);
        advance(u_tile, u_chunk_i, u_unit);
    }
    lds_barrier_wg();
    wrV ^= BUFSZ;
    read_b(0, 0, 0); read_b(1, 0, 1);

    // One unit = 4 runs of 8 MFMAs.  Gap r (before run r) reads the V operands of run
    // r+1 and reloads the A registers of run r-1 for unit i+1 (gap 0: those of run 3,
    // for unit i itself).  Gap 0 also holds the column half of the transform of unit
    // i+1 with six patch loads of unit i+2 between the pieces, gaps 1 and 2 the row
    // half (two pieces each) with the remaining loads, gap 3 the barrier.
    int cc = c_chunk;
    auto unit_body = [&]() {
        const int ukt = u_tile / a.tiles_t, ckt = c_tile / a.tiles_t;
        {
            const int before = x_tile;
            advance(x_tile, x_chunk_i, x_unit);
            if (x_tile != before) set_tile_block(x_tile % a.tiles_t);
        }
#pragma unroll
        for (int run = 0; run < 4; ++run) {
            const int cur = run & 1, nxt = cur ^ 1;
            const int p0 = (2 * run + 2) & 7, p1 = (2 * run + 3) & 7;
            const int q0 = (2 * run + 6) & 7, q1 = (2 * run + 7) & 7;
            if (run == 3) {
                lds_barrier_wg();
                flip();
            }
            read_b(p0, nxt, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (run == 0) load_a(q0, ckt, cc); else load_a(q0, ukt, u_chunk_i);
            __builtin_amdgcn_sched_barrier(0);
            read_b(p1, nxt, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (run == 0) load_a(q1, ckt, cc); else load_a(q1, ukt, u_chunk_i);
            __builtin_amdgcn_sched_barrier(0);
            // patch loads of unit i+2 (0-2 left dwords, 3-5 the 16-byte pieces, 6-8 right
            // dwords), each as soon as the transform has consumed its registers and a few
            // instructions away from the next load
            if (run == 0) {
                xform_col(0);
                __builtin_amdgcn_sched_barrier(0);
                load_x(0, x_chunk_i);
                __builtin_amdgcn_sched_barrier(0);
                xform_col(1);
                xform_col(2);
                __builtin_amdgcn_sched_barrier(0);
                load_x(1, x_chunk_i);
                __builtin_amdgcn_sched_barrier(0);
                xform_col(3);
                xform_col(4);
                __builtin_amdgcn_sched_barrier(0);
                load_x(2, x_chunk_i);
            } else if (run == 1) {
                xform_col(5);
                xform_row_store(0, 0);
                __builtin_amdgcn_sched_barrier(0);
                load_x(3, x_chunk_i);
                __builtin_amdgcn_sched_barrier(0);
                xform_row_store(0, 1);
                __builtin_amdgcn_sched_barrier(0);
                load_x(4, x_chunk_i);
            } else if (run == 2) {
                xform_row_store(1, 0);
                __builtin_amdgcn_sched_barrier(0);
                load_x(5, x_chunk_i);
                __builtin_amdgcn_sched_barrier(0);
                xform_row_store(1, 1);
                __builtin_amdgcn_sched_barrier(0);
                load_x(6, x_chunk_i);
            } else {
                load_x(7, x_chunk_i);
                __builtin_amdgcn_sched_barrier(0);
                load_x(8, x_chunk_i);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int u = q & 1, ks = q >> 1;
                acc[2 * run + u] = __builtin_amdgcn_mfma_f32_32x32x2f32(ar[2 * run + u][ks], bo[cur][u][ks],
                                                                         acc[2 * run + u], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        advance(u_tile, u_chunk_i, u_unit);
        ++cc;
    };

    // tile epilogue: partial output transform of this wave's two rows of M
    auto partial = [&](int v) -> floatx4 {
        float s0[4], s1[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float ma = acc[j][v], mb = acc[4 + j][v];      // rows 2*PH, 2*PH+1
            if (PH == 0) { s0[j] = ma + mb; s1[j] = mb; }
            else         { s0[j] = ma; s1[j] = -ma - mb; }
        }
        floatx4 y;
        y[0] = s0[0] + s0[1] + s0[2]; y[1] = s0[1] - s0[2] - s0[3];
        y[2] = s1[0] + s1[1] + s1[2]; y[3] = s1[1] - s1[2] - s1[3];
        return y;
    };
    auto finish_tile = [&](int tile_id, int first_unit) {
        const int kt = tile_id / a.tiles_t, tt = tile_id - kt * a.tiles_t;
        const bool head = first_unit < ub, tail = first_unit + nchunks > ue;
        // this wave finishes elements 8*PH .. 8*PH+7; the partner's partials for them
        // arrive through LDS, ours for the partner's elements go out the same way
        floatx4 *const xw = xchg + ((sub * 2 + PH) * 8) * 64 + lane;
        const floatx4 *const xrd = xchg + ((sub * 2 + (1 - PH)) * 8) * 64 + lane;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __builtin_amdgcn_sched_barrier(0);
            xw[e * 64] = partial(8 * (1 - PH) + e);
        }
        lds_barrier_wg();
        const int tile = tt * TB + wn0 + l32;
        const int tl = tile < a.T ? tile : 0;
        const int n = tl / (a.TH * a.TW), rem = tl - n * (a.TH * a.TW);
        const int th = rem / a.TW, tw = rem - th * a.TW;
        const int oh = 2 * th, ow = 2 * tw;
        const bool tv = tile < a.T && ow < a.Wout;
        const bool row1 = oh + 1 < a.Hout, col1 = ow + 1 < a.Wout;
        const int HWo = a.Hout * a.Wout;
        const int kbase = kt * KB + wm0 + 4 * lhi;
        float *ob = a.out + (int64_t)n * a.Kout * HWo + (int64_t)oh * a.Wout + ow + (int64_t)kbase * HWo;
        const float *bp = a.bias ? a.bias + kbase : nullptr;
        float *sp = a.partial + ((int64_t)lb * 2 + (head ? 0 : 1)) * (KB * TB * 4) +
                    ((wm0 + 4 * lhi) * TB + wn0 + l32) * 4;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __builtin_amdgcn_sched_barrier(0);
            const int v = 8 * PH + e;
            const int kr = 8 * (v >> 2) + (v & 3);
            floatx4 y = partial(v);
            const floatx4 o4 = xrd[e * 64];
            y[0] += o4[0]; y[1] += o4[1]; y[2] += o4[2]; y[3] += o4[3];
            if (head || tail) {
                *reinterpret_cast<floatx4 *>(sp + (kr * TB) * 4) = y;
            } else if (tv && kbase + kr < a.Kout) {
                const float bz = bp ? bp[kr] : 0.f;
                float *o = ob + (int64_t)kr * HWo;
                y[0] += bz; y[1] += bz; y[2] += bz; y[3] += bz;
                if (a.relu) { y[0] = fmaxf(y[0], 0.f); y[1] = fmaxf(y[1], 0.f); y[2] = fmaxf(y[2], 0.f); y[3] = fmaxf(y[3], 0.f); }
                if (a.pool) {
                    // one pooled pixel per tile (2x2 / stride-2 max pooling of the rectified output)
                    const int HWp = HWo >> 2;
                    a.out[((int64_t)n * a.Kout + kbase + kr) * HWp + th * (a.Wout >> 1) + tw] =
                        fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3]));
                } else if (a.vec2) {
                    *reinterpret_cast<float2 *>(o) = make_float2(y[0], y[1]);
                    if (row1) *reinterpret_cast<float2 *>(o + a.Wout) = make_float2(y[2], y[3]);
                } else {
                    o[0] = y[0];
                    if (col1) o[1] = y[1];
                    if (row1) {
                        o[a.Wout] = y[2];
                        if (col1) o[a.Wout + 1] = y[3];
                    }
                }
            }
        }
#pragma unroll
        for (int p = 0; p < 8; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;
    };

    int first_unit = ub - c_chunk;
    int i = 0;
    while (i < nunits) {
        int seg_end = i + (nchunks - c_chunk);
        if (seg_end > nunits) seg_end = nunits;
        for (; i < seg_end; ++i) unit_body();
        finish_tile(c_tile, first_unit);
        first_unit += nchunks;
        ++c_tile;
        c_chunk = 0;
        cc = 0;
    }
}

__global__ __launch_bounds__(512, 1) void wino_pair_kernel(WinoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // both halves run the same sequence of barriers
    if (threadIdx.x < 256) wino_pair_body<0, false>(a, lds);
    else wino_pair_body<1, false>(a, lds);
}

__global__ __launch_bounds__(512, 1) void wino_pair_ragged_kernel(WinoArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (threadIdx.x < 256) wino_pair_body<0, true>(a, lds);
    else wino_pair_body<1, true>(a, lds);
}

// Adds the two halves of every tile that a range boundary cut: boundary b lies
// between ranges b and b+1; tail slot of b + head slot of b+1 + bias -> y.
// Grid (G-1, 4): block (b, part) handles filters 16*part .. 16*part+15 of the cut
// tile; a thread keeps one tile column (its image coordinates are computed once)
// and walks over 4 filters.
__global__ __launch_bounds__(256) void wino_fixup_kernel(WinoArgs a, int G)
{
    constexpr int KB = kWinoKB, TB = kWinoTB;
    const int b = blockIdx.x;                 // boundary between logical ranges b and b+1
    const int unit = (int)((int64_t)(b + 1) * a.units_total / G);
    if (unit % a.nchunks == 0) return;        // boundary on a tile edge: nothing was cut
    const int tile_id = unit / a.nchunks;
    const int kt = tile_id / a.tiles_t, tt = tile_id - kt * a.tiles_t;
    const float *tailp = a.partial + ((int64_t)b * 2 + 1) * (KB * TB * 4);
    const float *headp = a.partial + ((int64_t)(b + 1) * 2 + 0) * (KB * TB * 4);
    const int HWo = a.Hout * a.Wout;
    const int tloc = threadIdx.x & 63;
    const int tile = tt * TB + tloc;
    if (tile >= a.T) return;
    const int n = tile / (a.TH * a.TW), rem = tile - n * (a.TH * a.TW);
    const int th = rem / a.TW, tw = rem - th * a.TW;
    const int oh = 2 * th, ow = 2 * tw;
    if (ow >= a.Wout) return;                 // phantom tile of a widened tile grid
    const bool row1 = oh + 1 < a.Hout, col1 = ow + 1 < a.Wout;
    float *obase = a.out + (int64_t)n * a.Kout * HWo + (int64_t)oh * a.Wout + ow;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int kl = blockIdx.y * 16 + (threadIdx.x >> 6) + 4 * i;
        const int k = kt * KB + kl;
        if (k >= a.Kout) continue;
        const int e = kl * TB + tloc;
        const floatx4 p = *reinterpret_cast<const floatx4 *>(tailp + e * 4);
        const floatx4 q = *reinterpret_cast<const floatx4 *>(headp + e * 4);
        const float bz = a.bias ? a.bias[k] : 0.f;
        float *o = obase + (int64_t)k * HWo;
        floatx4 y = {p[0] + q[0] + bz, p[1] + q[1] + bz, p[2] + q[2] + bz, p[3] + q[3] + bz};
        if (a.relu) { y[0] = fmaxf(y[0], 0.f); y[1] = fmaxf(y[1], 0.f); y[2] = fmaxf(y[2], 0.f); y[3] = fmaxf(y[3], 0.f); }
        if (a.pool) {
            const int HWp = HWo >> 2;
            a.out[((int64_t)n * a.Kout + k) * HWp + th * (a.Wout >> 1) + tw] = fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3]));
            continue;
        }
        o[0] = y[0];
        if (col1) o[1] = y[1];
        if (row1) {
            o[a.Wout] = y[2];
            if (col1) o[a.Wout + 1] = y[3];
        }
    }
}

int wino_filter_tile() { return kWinoKB; }
int wino_tile_block() { return kWinoTB; }
int wino_chan_chunk() { return kWinoCB; }
int wino_partial_slot_floats() { return kWinoKB * kWinoTB * 4; }

template <bool VEC>
static hipError_t launch_wino_variant(const WinoArgs &a, int G, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t cfg = hipSuccess;
    std::call_once(once, [] {
        cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_fused_kernel<VEC>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kWinoLdsBytes);
    });
    if (cfg != hipSuccess) return cfg;
    const ProfScope ps(KID_WINO_FUSED, 32.0 * a.T * (double)a.Cin * a.nsub * a.Kout,
                       (double)a.in_bytes + 4.0 * a.N * (double)a.Kout * a.Hout * a.Wout + 36.0 * a.Cin * (double)a.nsub * a.Kout, s);
    hipLaunchKernelGGL((wino_fused_kernel<VEC>), dim3((unsigned)G), dim3(256), kWinoLdsBytes, s, a);
    return hipGetLastError();
}

static hipError_t launch_wino_pair(const WinoArgs &a, int G, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t cfg = hipSuccess;
    std::call_once(once, [] {
        cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_pair_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kWinoPairLdsBytes);
        if (cfg == hipSuccess)
            cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_pair_ragged_kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kWinoPairLdsBytes);
    });
    if (cfg != hipSuccess) return cfg;
    const ProfScope ps(KID_WINO_PAIR, 32.0 * a.T * (double)a.Cin * a.Kout,
                       (double)a.in_bytes + 4.0 * a.N * (double)a.Kout * a.Hout * a.Wout + 36.0 * a.Cin * (double)a.Kout, s);
    if (a.Cin % kWinoCB != 0)
        hipLaunchKernelGGL(wino_pair_ragged_kernel, dim3((unsigned)G), dim3(512), kWinoPairLdsBytes, s, a);
    else
        hipLaunchKernelGGL(wino_pair_kernel, dim3((unsigned)G), dim3(512), kWinoPairLdsBytes, s, a);
    return hipGetLastError();
}

hipError_t launch_wino_fused(const WinoArgs &a, int G, hipStream_t s)
{
    hipError_t e;
    if (a.mode == 1) e = launch_wino_pair(a, G, s);
    else if (a.nsub > 1 || a.pad_w > 1 || a.Win % 2 != 0) e = launch_wino_variant<false>(a, G, s);
    else e = launch_wino_variant<true>(a, G, s);
    if (e != hipSuccess || G < 2) return e;
    // the fix-up pass is needed only if some range boundary falls inside a tile
    bool cut = false;
    for (int b = 0; b + 1 < G && !cut; ++b) cut = ((int64_t)(b + 1) * a.units_total / G) % a.nchunks != 0;
    if (!cut) return e;
    hipLaunchKernelGGL(wino_fixup_kernel, dim3((unsigned)(G - 1), 4), dim3(256), 0, s, a, G);
    return hipGetLastError();
}

}  // namespace mi355conv
