// Strided layers with large filters as stride-1 3x3 layers (first layers of AlexNet
// and Overfeat in Sec. 4.1 of the paper: 11x11, stride 4, 3 channels).
//
// With stride s and a filter of at most 3s x 3s taps, write a tap as r = s*r' + a,
// t = s*t' + b (r', t' in 0..2; a, b in 0..s-1).  Then
//   y[n,k,oh,ow] = sum_{c,r,t} w[k,c,r,t] * x[n,c, s*oh - pad_h + r, s*ow - pad_w + t]
//               = sum_{(a,b,c), r', t'} w2[k,(a,b,c),r',t'] * x2[n,(a,b,c), oh + r', ow + t']
// with the "space-to-depth" rearrangement
//   x2[n, (a*s + b)*C + c, i, j] = x[n, c, s*i + a - pad_h, s*j + b - pad_w]   (0 outside x)
//   w2[k, (a*s + b)*C + c, r', t'] = w[k, c, s*r' + a, s*t' + b]               (0 past the filter)
// i.e. an unpadded stride-1 3x3 layer over s*s*C channels on a (P+2) x (Q+2) map, which
// the Winograd kernels take: the gathers become contiguous, the matrix pipe sees s*s*C
// instead of C channels, and F(2x2,3x3) saves its 2.25x on top.  x2 is a permutation of
// the zero-padded x, so backward-data is the stride-1 backward-data into x2 followed by
// the inverse permutation, and backward-weight the stride-1 one followed by the inverse
// filter rearrangement.  Channels past s*s*C (x2 is padded to a multiple of the Winograd
// kernels' channel granularity) are zero.
//
// The four kernels here only move data; they are bound by HBM.

#include "conv_internal.h"

namespace mi355conv {

// A thread takes one (n, c, i, a, j): the s horizontally adjacent pixels b = 0..s-1 of x
// (consecutive addresses; consecutive lanes continue them, so a wave reads one contiguous
// run) go to s channel planes of x2 at the same (i, j) (a wave writes 64 consecutive floats
// per plane).  grid: x = ceil(s*H2*W2 / 256), y = C + 1, z = N; y == C clears the padding
// channels s*s*C .. Cq-1 of image n.
template <int S>
__global__ __launch_bounds__(256) void space_to_depth_kernel(S2dArgs a)
{
    const int n = blockIdx.z;
    const int plane = a.H2 * a.W2;
    if ((int)blockIdx.y == a.C) {
        const int64_t cnt = (int64_t)(a.Cq - S * S * a.C) * plane;
        float *dst = a.x2 + ((int64_t)n * a.Cq + S * S * a.C) * plane;
        for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < cnt; t += (int64_t)gridDim.x * 256) dst[t] = 0.f;
        return;
    }
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= S * plane) return;
    const int c = blockIdx.y;
    const int ia = (int)fast_div((uint32_t)idx, a.div_W2), j = idx - ia * a.W2;     // ia = i*S + a
    const int i = ia / S, ra = ia - i * S;
    const int h = ia - a.pad_h, w0 = S * j - a.pad_w;
    const bool hv = (unsigned)h < (unsigned)a.H;
    const float *src = a.x + (((int64_t)n * a.C + c) * a.H + (hv ? h : 0)) * a.W;
    float *dst = a.x2 + (((int64_t)n * a.Cq + (int64_t)(ra * S) * a.C + c) * a.H2 + i) * a.W2 + j;
#pragma unroll
    for (int b = 0; b < S; ++b) {
        const int w = w0 + b;
        dst[(int64_t)b * a.C * plane] = (hv && (unsigned)w < (unsigned)a.W) ? src[w] : 0.f;
    }
}

// Inverse permutation, same thread assignment: reads s planes of x2 at (i, j), writes s
// adjacent pixels of dx.  The (i, j) range is extended so that every pixel of dx is written;
// pixels no window reaches have no source in x2 and get 0.  grid: x = ceil(S*I2*J2 / 256),
// y = C, z = N with I2 = max(H2, ceil((H + pad_h) / S)), J2 likewise.
template <int S>
__global__ __launch_bounds__(256) void depth_to_space_kernel(S2dArgs a)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= S * a.I2 * a.J2) return;
    const int c = blockIdx.y, n = blockIdx.z;
    const int plane = a.H2 * a.W2;
    const int ia = (int)fast_div((uint32_t)idx, a.div_J2), j = idx - ia * a.J2;
    const int i = ia / S, ra = ia - i * S;
    const int h = ia - a.pad_h, w0 = S * j - a.pad_w;
    if ((unsigned)h >= (unsigned)a.H) return;
    const bool sv = i < a.H2 && j < a.W2;
    const float *src = a.x2 + (((int64_t)n * a.Cq + (int64_t)(ra * S) * a.C + c) * a.H2 + (sv ? i : 0)) * a.W2 + (sv ? j : 0);
    float *dst = a.dx + (((int64_t)n * a.C + c) * a.H + h) * a.W;
#pragma unroll
    for (int b = 0; b < S; ++b) {
        const int w = w0 + b;
        if ((unsigned)w < (unsigned)a.W) dst[w] = sv ? src[(int64_t)b * a.C * plane] : 0.f;
    }
}

// w [K][C][R][S] -> w2 [K][Cq][3][3]; one thread per element of w2
__global__ __launch_bounds__(256) void filter_s2d_kernel(const float *__restrict__ w, float *__restrict__ w2,
                                                         int K, int C, int R, int S, int s, int Cq)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * Cq * 9) return;
    const int t2 = idx % 3, r2 = (idx / 3) % 3, cq = (idx / 9) % Cq, k = idx / (9 * Cq);
    float v = 0.f;
    if (cq < s * s * C) {
        const int ab = cq / C, c = cq - ab * C, ra = ab / s, rb = ab - ra * s;
        const int r = s * r2 + ra, t = s * t2 + rb;
        if (r < R && t < S) v = w[(((int64_t)k * C + c) * R + r) * S + t];
    }
    w2[idx] = v;
}

// dw[k][c][r][t] = dw2[k][(a*s + b)*C + c][r'][t'] (+ dw): one thread per element of dw
__global__ __launch_bounds__(256) void filter_d2s_kernel(const float *__restrict__ dw2, float *__restrict__ dw,
                                                         int K, int C, int R, int S, int s, int Cq, int accumulate)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * C * R * S) return;
    const int t = idx % S, r = (idx / S) % R, c = (idx / (S * R)) % C, k = idx / (S * R * C);
    const int r2 = r / s, ra = r - r2 * s, t2 = t / s, rb = t - t2 * s;
    const float v = dw2[(((int64_t)k * Cq + (ra * s + rb) * C + c) * 3 + r2) * 3 + t2];
    dw[idx] = accumulate ? dw[idx] + v : v;
}

hipError_t launch_space_to_depth(const S2dArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)((a.s * a.H2 * a.W2 + 255) / 256), (unsigned)(a.C + 1), (unsigned)a.N);
    switch (a.s) {
    case 2: hipLaunchKernelGGL(space_to_depth_kernel<2>, grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL(space_to_depth_kernel<3>, grid, dim3(256), 0, s, a); break;
    case 4: hipLaunchKernelGGL(space_to_depth_kernel<4>, grid, dim3(256), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_depth_to_space(const S2dArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)((a.s * a.I2 * a.J2 + 255) / 256), (unsigned)a.C, (unsigned)a.N);
    switch (a.s) {
    case 2: hipLaunchKernelGGL(depth_to_space_kernel<2>, grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL(depth_to_space_kernel<3>, grid, dim3(256), 0, s, a); break;
    case 4: hipLaunchKernelGGL(depth_to_space_kernel<4>, grid, dim3(256), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_filter_s2d(const float *w, float *w2, int K, int C, int R, int S, int stride, int Cq,
                             hipStream_t s)
{
    const int total = K * Cq * 9;
    hipLaunchKernelGGL(filter_s2d_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, w2, K, C,
                       R, S, stride, Cq);
    return hipGetLastError();
}

hipError_t launch_filter_d2s(const float *dw2, float *dw, int K, int C, int R, int S, int stride, int Cq,
                             int accumulate, hipStream_t s)
{
    const int total = K * C * R * S;
    hipLaunchKernelGGL(filter_d2s_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, dw2, dw, K, C,
                       R, S, stride, Cq, accumulate);
    return hipGetLastError();
}

}  // namespace mi355conv
