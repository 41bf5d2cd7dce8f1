// Frequency-domain convolution (Sec. 4.2 "fft": the layer as a product of spectra, the
// choice for large filters such as 5x5) for stride-1 layers whose padded input fits ONE
// 32 x 32 tile per image (27x27 + 2x2, 28x28 + 0, 28x28 + 2x2: the 5x5 layers of the AlexNet,
// Overfeat and inception configurations).  With one tile per image there is no overlap-add:
// a circular correlation of length 32 has no wrap-around in the outputs that are kept.
//
//   X[f][n][c] = DFT of the image (n, c) placed at (pad_h, pad_w) of a zero tile     (fft_image_kernel)
//   A[f][c][k] = conj(DFT of the filter (k, c), zero-extended): the same kernel, the
//                filter being an R x S image                                         (fft_image_kernel)
//   M[f][n][k] = sum_c X[f][n][c] A[f][c][k]     one complex GEMM per frequency      (wino4_gemm_kernel)
//   y[n][k]    = inverse DFT of M[.][n][k], rows and columns < P, Q, + bias          (fft_inverse_kernel)
//
// Backward-data is the same with dy at (0, 0), the filter spectrum unconjugated and k <-> c
// swapped, and the rows and columns pad .. pad + H - 1 of the inverse kept.  Backward-weight
// takes the images as the GEMM's depth: G[f][k][c] = sum_n dY[f][k][n] conj(X[f][c][n]), and
// the R x S corner of the inverse of conj(G) is the filter gradient (the same inverse kernel
// with "image" (k, c)); the bias gradient is the zero frequency of dY summed over the images.
//
// Real input: only the rows u = 0..16 of the spectrum are kept (the others are conjugates),
// 544 frequencies f = v * 17 + u.  The complex products run on the real fp32 GEMM of the
// Winograd F(4x4,3x3) path: the operand on the column side becomes the real matrix with
// columns 2m + po and depth 2d + pi, [Ar -Ai; Ai Ar], the other one the stacked (re, im)
// pairs along the depth; a result row then holds (re, im) pairs of neighbouring channels, which
// the inverse kernel gathers as whole 128-byte lines.
//
// The transforms are dense 32-point DFT matrices on the matrix cores, not butterflies: a
// 32 x 32 tile takes 48 v_mfma_f32_32x32x2_f32 (82 for the inverse), a wave per image, and the
// data never leaves the registers between the two passes: the accumulator layout of the
// first product (lane = column, registers = rows) is the B-operand layout of the second, whose
// reduction runs over those rows in the order the registers hold them (the constant A operand
// is permuted to match).  Error against the oracle: 2e-7 .. 4e-7 of max|ref|, each output
// being a sum of 32-term dot products with fp32 sines and cosines.

#include "conv_internal.h"

#include <mutex>

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kUH = 17, kF = kFftFreqs;      // kept rows of a 32 x 32 spectrum; kept frequencies

// row of accumulator element e in a lane of the upper (hi = 1) or lower half of the wave
__device__ __forceinline__ int acc_row(int e, int hi) { return 8 * (e >> 2) + 4 * hi + (e & 3); }

// cos and sin of 2 pi m / 32 from a 64-float table in LDS (cosines, then sines), filled by the
// first 32 threads of the workgroup: a wave needs ~60 of them for four images, and computing
// each one costs as much as several MFMAs
__device__ __forceinline__ void cs32_fill(float *tab)
{
    if (threadIdx.x < 32) sincospif((float)threadIdx.x * (1.f / 16.f), &tab[32 + threadIdx.x], &tab[threadIdx.x]);
    __syncthreads();
}
__device__ __forceinline__ void cs32(const float *tab, int m, float &c, float &s) { c = tab[m & 31]; s = tab[32 + (m & 31)]; }

// ------------------------------------------------------------------ images
// One wave per (b, four consecutive a): image (a, b) at in + a * stride_a + b * stride_b.
// Forward / backward-data: a = reduction channel, b = image; for the filters a = the reduced
// axis of w, b = the other one.  Backward-weight: a = image, b = channel (x) or filter (dy).
// Output dst[chunk][half][f][row][4]: the frequency is not the slowest index, so what one
// workgroup writes (and what an inverse workgroup gathers from the products, laid out the same
// way) lies a row pitch apart per frequency, within about a megabyte, instead of a whole operand
// slice apart.  Inside an 8-deep chunk the four images a and their two parts sit as
// [half = a % 2][row][2 * ((a % 4) / 2) + part]: a 16-byte vector holds the (re, im) pairs of the
// images a and a + 2, so a wave takes its images in the order 0, 2 (half 0), then 1, 3 (half 1)
// and hands a finished pair to the staging area (any order of the depth serves, as long as both
// operands use the same).
//   mode 0: row b: (re, im)                                    (stacked pairs, b as row)
//   mode 1: conjugate in block form, columns 2b + po: column 2b: (re, im), column 2b+1: (-im, re)
//   mode 2: block form of the spectrum itself:        column 2b: (re, -im), column 2b+1: (im, re)
// a >= na: zeros (the depth is padded to a multiple of 4 with zeros in both operands).
// The steps of the first pass whose two tile rows lie outside the image are skipped (a 5 x 5
// filter has 3 of 16).
struct FftImgArgs {
    const float *in;
    float *dst;
    int32_t in_bytes;
    int32_t na, nb, stride_a, stride_b;     // strides in floats
    int32_t H, W, off_h, off_w;
    int32_t chunks, pitch, mode;
};

// Staging area of a workgroup: per frequency one 128-byte line of the operand (8 rows of 16
// bytes) + 16 bytes so that the lanes of a wave, which hold neighbouring frequencies, hit
// different banks; then the 64-float sine / cosine table.
constexpr int kStageF = 36;                                  // floats per frequency
constexpr int kImgLds = (kF * kStageF + 64) * 4;

// ROWS operand rows per image b: 1 (mode 0: a workgroup of 8 waves takes 8 images b, so that a
// compute unit holds two waves per SIMD in ONE workgroup and the launch splits into many short
// rounds) or 2 (block form: 4 waves, 4 images b, columns 2b and 2b + 1).  Every
// half-chunk is staged in LDS and leaves as whole 128-byte lines: a compute unit completes
// about one line-sized store per ~20 cycles, and a wave storing its own 16-byte pieces asks for
// 34 different lines per instruction (the kernel's time was then set by the number of its stores).
template <int ROWS, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 512 / (64 * WAVES)) void fft_image_kernel(FftImgArgs a)
{
    extern __shared__ float sm[];
    float *tab = sm + kF * kStageF;
    cs32_fill(tab);
    constexpr int NB = 8 / ROWS, ROUNDS = NB / WAVES;        // images b per workgroup; per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b0 = blockIdx.x * NB;
    const int chunk = blockIdx.y;
    const int l32 = lane & 31, hi = lane >> 5;
    // first pass: Z^T[w][u] = sum_h X[h][w] exp(-2 pi i h u / 32); B operand [k = h][col].  The
    // input is real, so Z[0] and Z[16] are real: Re Z[u], u = 0..16, and Im Z[u], u = 1..15, are
    // exactly 32 columns, col = u and col = 16 + u, and ONE product gives both.
    // second pass: sum_w exp(-2 pi i w v / 32) Z^T[w][u] = (C - iS)(Zr + iZi); A operand [row = v]
    // [k = w], w in the order the accumulators of the first pass hold their rows; P1 = C . Zp and
    // P2 = S . Zp on the packed columns, then Yr[u] = P1[u] + P2[16 + u], Yi[u] = P1[16 + u] - P2[u]
    // with one exchange between the lanes u and 16 + u per register.
    float c1[16], c2[16], s2[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        float c, sn;
        cs32(tab, (2 * s + hi) * (l32 <= 16 ? l32 : l32 - 16), c, sn);
        c1[s] = l32 <= 16 ? c : -sn;
        cs32(tab, acc_row(s, hi) * l32, c, sn);
        c2[s] = c; s2[s] = sn;
    }
    const float pm = (l32 >= 1 && l32 <= 15) ? 1.f : 0.f;    // the lanes u that have an imaginary column
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, a.in_bytes, 0x00020000);
    // A operand of the first pass: lane = column w of the tile, step s = rows 2s + hi; the
    // image's own offset (a, b: uniform in the wave) goes into the scalar offset
    const int col = l32 - a.off_w;
    const bool colok = (unsigned)col < (unsigned)a.W;
    uint32_t off[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const int row = 2 * s + hi - a.off_h;
        off[s] = colok && (unsigned)row < (unsigned)a.H ? (uint32_t)((row * a.W + col) * 4) : 0x80000000u;
    }
    const int s_lo = a.off_h >> 1, s_hi = (a.off_h + a.H + 1) >> 1;     // steps 2s, 2s+1 that touch the image's rows
    // the wave's images in the order it takes them: (half, round, first / second of the pair);
    // image a = 4 * chunk + half + 2 * second of b = b0 + WAVES * round + wave
    float x[16];
    auto load_x = [&](int seq) {
        const int second = seq & 1, round = (seq >> 1) % ROUNDS, half = (seq >> 1) / ROUNDS;
        const int ai = chunk * 4 + half + 2 * second, b = b0 + WAVES * round + wave;
        const bool ok = ai < a.na && b < a.nb;
        const uint32_t bad = ok ? 0u : 0x80000000u;
        const int so = ok ? (ai * a.stride_a + b * a.stride_b) * 4 : 0;
#pragma unroll
        for (int s = 0; s < 16; ++s) x[s] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off[s] | bad, so, 0));
    };
    load_x(0);
    const int64_t fstride = (int64_t)a.pitch * 4;            // floats between frequencies
    floatx16 pr, pi;                                         // the first image of a pair
#pragma unroll
    for (int seq = 0; seq < 4 * ROUNDS; ++seq) {
        const int second = seq & 1, round = (seq >> 1) % ROUNDS, half = (seq >> 1) / ROUNDS;
        floatx16 z, p1, p2, yr, yi;
#pragma unroll
        for (int e = 0; e < 16; ++e) { z[e] = 0.f; p1[e] = 0.f; p2[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            if (s >= s_lo && s < s_hi)                       // uniform
                z = __builtin_amdgcn_mfma_f32_32x32x2f32(x[s], c1[s], z, 0, 0, 0);
        }
        // the first pass has read x: the next image's loads go out here and are in flight during
        // the 32 MFMAs of the second pass
        __builtin_amdgcn_sched_barrier(0);
        if (seq + 1 < 4 * ROUNDS) load_x(seq + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            p1 = __builtin_amdgcn_mfma_f32_32x32x2f32(c2[s], z[s], p1, 0, 0, 0);
            p2 = __builtin_amdgcn_mfma_f32_32x32x2f32(s2[s], z[s], p2, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float q1 = __shfl_xor(p1[e], 16), q2 = __shfl_xor(p2[e], 16);
            yr[e] = p1[e] + pm * q2;
            yi[e] = pm * q1 - p2[e];
        }
        if (!second) {
            pr = yr; pi = yi;
            continue;
        }
        // the pair's spectra into the staging line of their frequency: lane = u (kept below 17),
        // element e = row v; slot = the operand row inside the workgroup's 8
        if (l32 < kUH) {
            const int slot = (WAVES * round + wave) * ROWS;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float *q = sm + (acc_row(e, hi) * kUH + l32) * kStageF + slot * 4;
                if (ROWS == 1) {
                    const floatx4 v = {pr[e], pi[e], yr[e], yi[e]};
                    *reinterpret_cast<floatx4 *>(q) = v;
                } else {
                    const float sg = a.mode == 1 ? 1.f : -1.f;
                    const floatx4 v0 = {pr[e], sg * pi[e], yr[e], sg * yi[e]};
                    const floatx4 v1 = {-sg * pi[e], pr[e], -sg * yi[e], yr[e]};
                    *reinterpret_cast<floatx4 *>(q) = v0;
                    *reinterpret_cast<floatx4 *>(q + 4) = v1;
                }
            }
        }
        if (round == ROUNDS - 1) {
            // the half-chunk is complete: out as whole lines (thread t: 16 bytes of line f)
            __syncthreads();
            const int row0 = b0 * ROWS, nrows = a.nb * ROWS;
            float *base = a.dst + ((int64_t)chunk * 2 + half) * kF * fstride + (int64_t)row0 * 4;
#pragma unroll
            for (int i = 0; i < (kF * 8 + 64 * WAVES - 1) / (64 * WAVES); ++i) {
                const int idx = threadIdx.x + 64 * WAVES * i, f = idx >> 3, r8 = idx & 7;
                if (idx < kF * 8 && row0 + r8 < nrows)
                    *reinterpret_cast<floatx4 *>(base + (int64_t)f * fstride + r8 * 4) =
                        *reinterpret_cast<const floatx4 *>(sm + f * kStageF + r8 * 4);
            }
            __syncthreads();
        }
    }
}

// ------------------------------------------------------------------ inverse
// "Image" (row, ch) of the products M[row][f][2 ch + po] (a row's frequencies next to each
// other): forward (n, k), backward-data (n, c), backward-weight (k, c).  A workgroup takes the 16 channels ch0 .. ch0 + 15 of one row: per
// frequency their 32 values are one 128-byte line of M; the 544 lines are gathered into LDS
// ([channel][part * 544 + f], channel stride 1089 floats), then every wave transforms four
// images.
//   T[u][q] = sum_v Y[u][v] exp(+2 pi i v q / 32)              A operand = Y (lane = u, step = v)
//   y[p][q] = sum_{u<17} Gc[p][u] Tr[u][q] + Gs[p][u] Ti[u][q]   Gc = wu cos / 1024, Gs = -wu sin / 1024,
//                                                               wu = 1, 2, ..., 2, 1
// out[((row * nch + ch) * Hout + p - off_h) * Wout + q - off_w] = scale * y[p][q] (+ bias[ch], rectifier,
// or + the old value); conj: the inverse of the conjugate spectrum.
struct FftInvArgs {
    const float *M;
    const float *bias;         // nullable, per channel
    float *out;
    int32_t nrow, nch, Hout, Wout, off_h, off_w;
    int32_t Npad;              // columns of M per row and frequency
    int32_t relu, conj, accumulate;
    float scale;
};
constexpr int kInvImages = 16, kInvStride = 2 * kF + 1;
constexpr int kInvLds = (kInvImages * kInvStride + 64) * 4;          // + the sine / cosine table

__global__ __launch_bounds__(256) void fft_inverse_kernel(FftInvArgs a)
{
    extern __shared__ float sm[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int ch0 = blockIdx.x * kInvImages, row = blockIdx.y;
    {
        // thread t: frequency (t / 8) + 32 * pass, values 4 * (t % 8) .. + 3 of its line
        const int q8 = threadIdx.x & 7;
        const int f0 = threadIdx.x >> 3;
        const float *src = a.M + ((int64_t)row * kF + f0) * a.Npad + 2 * ch0 + 4 * q8;
        const int64_t step = (int64_t)32 * a.Npad;
        floatx4 v[17];                        // all 17 loads issued before the first store: one memory latency, not 17
#pragma unroll
        for (int i = 0; i < 17; ++i) v[i] = *reinterpret_cast<const floatx4 *>(src + i * step);
        float *d = sm + (2 * q8) * kInvStride + f0;
#pragma unroll
        for (int i = 0; i < 17; ++i) {
            d[32 * i] = v[i][0];                      // channel 2 q8, re
            d[32 * i + kF] = v[i][1];                 //               im
            d[32 * i + kInvStride] = v[i][2];         // channel 2 q8 + 1
            d[32 * i + kInvStride + kF] = v[i][3];
        }
    }
    float *tab = sm + kInvImages * kInvStride;
    cs32_fill(tab);                           // its barrier also covers the gather
    float ce[16], se[16], gc[9], gs[9];
#pragma unroll
    for (int s = 0; s < 16; ++s) cs32(tab, (2 * s + hi) * l32, ce[s], se[s]);
#pragma unroll
    for (int s = 0; s < 9; ++s) {
        const int u = acc_row(s, hi);
        float c, sn;
        cs32(tab, u * l32, c, sn);
        const float wu = u > 16 ? 0.f : (u == 0 || u == 16) ? 1.f / 1024.f : 2.f / 1024.f;
        gc[s] = wu * c;
        gs[s] = -wu * sn;
    }
    const float sgn = a.conj ? -1.f : 1.f;
    for (int i = 0; i < 4; ++i) {
        const int img = wave * 4 + i, ch = ch0 + img;
        if (ch >= a.nch) break;                              // uniform in the wave
        const float *y = sm + img * kInvStride;
        floatx16 tr, ti, o;
#pragma unroll
        for (int e = 0; e < 16; ++e) { tr[e] = 0.f; ti[e] = 0.f; o[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int f = (2 * s + hi) * kUH + l32;
            const float yr = l32 < kUH ? y[f] : 0.f, yi = l32 < kUH ? sgn * y[kF + f] : 0.f;
            tr = __builtin_amdgcn_mfma_f32_32x32x2f32(yr, ce[s], tr, 0, 0, 0);
            tr = __builtin_amdgcn_mfma_f32_32x32x2f32(-yi, se[s], tr, 0, 0, 0);
            ti = __builtin_amdgcn_mfma_f32_32x32x2f32(yr, se[s], ti, 0, 0, 0);
            ti = __builtin_amdgcn_mfma_f32_32x32x2f32(yi, ce[s], ti, 0, 0, 0);
        }
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            o = __builtin_amdgcn_mfma_f32_32x32x2f32(gc[s], tr[s], o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_32x32x2f32(gs[s], ti[s], o, 0, 0, 0);
        }
        // lane = column q of the tile, element e = row
        const int q = l32 - a.off_w;
        const float bz = a.bias ? a.bias[ch] : 0.f;
        float *dst = a.out + ((int64_t)row * a.nch + ch) * a.Hout * a.Wout;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int p = acc_row(e, hi) - a.off_h;
            if ((unsigned)p < (unsigned)a.Hout && (unsigned)q < (unsigned)a.Wout) {
                float val = a.scale * o[e] + bz;
                if (a.relu) val = fmaxf(val, 0.f);
                if (a.accumulate) val += dst[p * a.Wout + q];
                dst[p * a.Wout + q] = val;
            }
        }
    }
}

// db[k] = sum over the images of the zero frequency (real part) of dY, A[chunk][a % 2][f = 0][k][..]
__global__ __launch_bounds__(256) void fft_wg_bias_kernel(FftWgradArgs a)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= a.K) return;
    float sacc = 0.f;
    for (int chunk = 0; chunk < a.chunks; ++chunk) {
        // the real parts of the chunk's four images: elements 0 and 2 of both halves
        const floatx4 v = *reinterpret_cast<const floatx4 *>(a.A + ((int64_t)chunk * 2 * kF * a.Mpad + k) * 4);
        const floatx4 w = *reinterpret_cast<const floatx4 *>(a.A + ((int64_t)(chunk * 2 + 1) * kF * a.Mpad + k) * 4);
        sacc += (v[0] + w[0]) + (v[2] + w[2]);
    }
    const float g = a.scale * sacc;
    a.db[k] = a.accumulate ? a.db[k] + g : g;
}

// the GEMM over all frequencies: whole rounds one workgroup per tile, the tiles of the last,
// partly filled round as depth shares + fix-up (as in the Winograd F(4x4,3x3) path)
hipError_t run_gemm(const float *A, const float *B, float *M, float *slots, int chunks, int Mpad, int Npad, int cfg,
                    int split, int split_tiles, double flops, double bytes, hipStream_t s)
{
    W4GemmArgs g = {};
    g.A = A; g.B = B; g.C = M;
    g.chunks = chunks; g.Mpad = Mpad; g.Npad = Npad;
    g.tiles_m = Mpad / wino4_tile_m(cfg);
    g.tiles_n = Npad / wino4_tile_n(cfg);
    g.batch_inner = 1;                       // operands [chunk][half][f][row][4], products [row][f][col]
    const int tiles = kF * g.tiles_m * g.tiles_n;
    const int full = split > 1 ? tiles - split_tiles : tiles;
    hipError_t e = hipSuccess;
    if (full > 0) {
        g.tile_base = 0; g.nsplit = 1;
        const ProfScope ps(KID_WINO4_GEMM, flops * full / tiles, bytes * full / tiles, s);
        launch_w4_gemm(g, cfg, (unsigned)full, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (full < tiles) {
        g.tile_base = full; g.nsplit = split; g.slots = slots;
        {
            const ProfScope ps(KID_WINO4_GEMM, flops * (tiles - full) / tiles, bytes * (tiles - full) / tiles, s);
            launch_w4_gemm(g, cfg, (unsigned)((tiles - full) * split), s);
            e = hipGetLastError();
        }
        if (e != hipSuccess) return e;
        launch_w4_fixup(g, cfg, (unsigned)(tiles - full), s);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_image(const FftImgArgs &ia, int kid, hipStream_t s)
{
    const int steps = ((ia.off_h + ia.H + 1) >> 1) - (ia.off_h >> 1);
    const ProfScope ps(kid, (steps + 32.0) * 4096.0 * ia.nb * (double)ia.chunks * 4,
                       (double)ia.in_bytes + 4.0 * kF * ia.chunks * 8.0 * ia.nb * (ia.mode ? 2 : 1), s);
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(fft_image_kernel<1, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, kImgLds);
        if (attr == hipSuccess)
            attr = hipFuncSetAttribute(reinterpret_cast<const void *>(fft_image_kernel<2, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, kImgLds);
    });
    if (attr != hipSuccess) return attr;
    if (ia.mode == 0)
        hipLaunchKernelGGL((fft_image_kernel<1, 8>), dim3((unsigned)((ia.nb + 7) / 8), (unsigned)ia.chunks), dim3(512), kImgLds, s, ia);
    else
        hipLaunchKernelGGL((fft_image_kernel<2, 4>), dim3((unsigned)((ia.nb + 3) / 4), (unsigned)ia.chunks), dim3(256), kImgLds, s, ia);
    return hipGetLastError();
}

hipError_t launch_inverse(const FftInvArgs &ia, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(fft_inverse_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kInvLds);
    });
    if (attr != hipSuccess) return attr;
    const ProfScope ps(KID_FFT_INVERSE, 82.0 * 4096.0 * ia.nrow * (double)ia.nch,
                       8.0 * kF * ia.nrow * (double)ia.nch + 4.0 * ia.nrow * (double)ia.nch * ia.Hout * ia.Wout, s);
    hipLaunchKernelGGL(fft_inverse_kernel, dim3((unsigned)((ia.nch + kInvImages - 1) / kInvImages), (unsigned)ia.nrow), dim3(256),
                       kInvLds, s, ia);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fft_conv(const FftArgs &a, hipStream_t s)
{
    const int RS = a.R * a.S;
    // column side: the filters as R x S images; forward: conj(W[k][c]) with depth c, columns k;
    // backward-data: W[k][c] with depth k, columns c
    FftImgArgs fw = {};
    fw.in = a.w; fw.dst = a.B; fw.in_bytes = a.w_bytes;
    fw.na = a.Cin; fw.nb = a.Kout;
    fw.stride_a = a.mode == 0 ? RS : a.C * RS; fw.stride_b = a.mode == 0 ? a.C * RS : RS;
    fw.H = a.R; fw.W = a.S; fw.off_h = 0; fw.off_w = 0;
    fw.chunks = a.chunks; fw.pitch = a.Npad; fw.mode = a.mode == 0 ? 1 : 2;
    hipError_t e = launch_image(fw, KID_FFT_FILTER, s);
    if (e != hipSuccess) return e;
    // row side: the images
    FftImgArgs ia = {};
    ia.in = a.in; ia.dst = a.A; ia.in_bytes = a.in_bytes;
    ia.na = a.Cin; ia.nb = a.N; ia.stride_a = a.Hin * a.Win; ia.stride_b = a.Cin * a.Hin * a.Win;
    ia.H = a.Hin; ia.W = a.Win; ia.off_h = a.in_off_h; ia.off_w = a.in_off_w;
    ia.chunks = a.chunks; ia.pitch = a.Mpad; ia.mode = 0;
    e = launch_image(ia, KID_FFT_IMAGE, s);
    if (e != hipSuccess) return e;
    const double a_b = 4.0 * kF * a.chunks * 8.0 * a.Mpad, b_b = 4.0 * kF * a.chunks * 8.0 * a.Npad, m_b = 4.0 * kF * a.Mpad * (double)a.Npad;
    e = run_gemm(a.A, a.B, a.M, a.slots, a.chunks, a.Mpad, a.Npad, a.tile_cfg, a.split, a.split_tiles,
                 8.0 * kF * a.Kout * (double)a.Cin * a.N, a_b + b_b + m_b, s);
    if (e != hipSuccess) return e;
    FftInvArgs iv = {};
    iv.M = a.M; iv.bias = a.bias; iv.out = a.out;
    iv.nrow = a.N; iv.nch = a.Kout; iv.Hout = a.Hout; iv.Wout = a.Wout; iv.off_h = a.out_off_h; iv.off_w = a.out_off_w;
    iv.Npad = a.Npad; iv.relu = a.relu; iv.conj = 0; iv.accumulate = 0; iv.scale = 1.f;
    return launch_inverse(iv, s);
}

hipError_t launch_fft_wgrad(const FftWgradArgs &a, hipStream_t s)
{
    // row side: dY[k][n], depth n; column side: conj(X[c][n]) in block form
    FftImgArgs iy = {};
    iy.in = a.dy; iy.dst = a.A; iy.in_bytes = a.dy_bytes;
    iy.na = a.N; iy.nb = a.K; iy.stride_a = a.K * a.P * a.Q; iy.stride_b = a.P * a.Q;
    iy.H = a.P; iy.W = a.Q; iy.off_h = 0; iy.off_w = 0;
    iy.chunks = a.chunks; iy.pitch = a.Mpad; iy.mode = 0;
    hipError_t e = launch_image(iy, KID_FFT_IMAGE, s);
    if (e != hipSuccess) return e;
    FftImgArgs ix = {};
    ix.in = a.x; ix.dst = a.B; ix.in_bytes = a.x_bytes;
    ix.na = a.N; ix.nb = a.C; ix.stride_a = a.C * a.H * a.W; ix.stride_b = a.H * a.W;
    ix.H = a.H; ix.W = a.W; ix.off_h = a.pad_h; ix.off_w = a.pad_w;
    ix.chunks = a.chunks; ix.pitch = a.Npad; ix.mode = 1;
    e = launch_image(ix, KID_FFT_IMAGE, s);
    if (e != hipSuccess) return e;
    const double a_b = 4.0 * kF * a.chunks * 8.0 * a.Mpad, b_b = 4.0 * kF * a.chunks * 8.0 * a.Npad, m_b = 4.0 * kF * a.Mpad * (double)a.Npad;
    e = run_gemm(a.A, a.B, a.M, a.slots, a.chunks, a.Mpad, a.Npad, a.tile_cfg, a.split, a.split_tiles,
                 8.0 * kF * a.K * (double)a.C * a.N, a_b + b_b + m_b, s);
    if (e != hipSuccess) return e;
    // the filter gradient: the R x S corner of the inverse of conj(G[k][c])
    FftInvArgs iv = {};
    iv.M = a.M; iv.bias = nullptr; iv.out = a.dw;
    iv.nrow = a.K; iv.nch = a.C; iv.Hout = a.R; iv.Wout = a.S; iv.off_h = 0; iv.off_w = 0;
    iv.Npad = a.Npad; iv.relu = 0; iv.conj = 1; iv.accumulate = a.accumulate; iv.scale = a.scale;
    e = launch_inverse(iv, s);
    if (e != hipSuccess || !a.db) return e;
    hipLaunchKernelGGL(fft_wg_bias_kernel, dim3((unsigned)((a.K + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace mi355conv
