// Backward-data of a first layer: 3x3, stride 1, very few input channels (C <= 4).
//
// With C = 3 the GEMM form of backward-data has only 3 useful rows out of a
// 32-row MFMA tile, so the matrix pipe cannot be used sensibly; the layer is
// bound by reading dy once (Sec. 4.1 of the paper times such layers as part of
// the convolution stack although frameworks usually skip this gradient).  This
// kernel computes it directly on the vector ALU:
//   dx[n,c,h,v] = sum_{k,r,s} dy[n,k,h+pad_h-r,v+1-s] * w[k,c,r,s]
// Each thread owns 4 consecutive pixels of one row for all C channels.  Per
// (k, r) it fetches the 6 values of dy it needs with three buffer loads whose
// per-thread offsets are fixed (left neighbour, aligned 16 bytes, right
// neighbour; k advances through the scalar offset; rows or neighbours outside
// the image carry an offset beyond the buffer and read as 0) and does 12*C
// multiply-adds whose weight operand is a scalar register (the weights of one k
// are 9*C consecutive floats of w, fetched with scalar loads).

#include "conv_internal.h"

namespace mi355conv {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int C>
__global__ __launch_bounds__(256) void bwd_data_smallc_kernel(SmallCArgs a)
{
    const int quads_per_row = a.W >> 2;
    const int64_t total = (int64_t)a.N * a.H * quads_per_row;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool tv = t < total;
    const int64_t tt = tv ? t : 0;
    const int qd = (int)(tt % quads_per_row);
    const int h = (int)((tt / quads_per_row) % a.H);
    const int n = (int)(tt / ((int64_t)quads_per_row * a.H));
    const int v0 = qd * 4;

    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.dy_bytes, 0x00020000);
    const int PQ = a.P * a.Q;
    // fixed byte offsets inside filter plane 0 of image n: rows p = h + pad_h - r
    uint32_t off_l[3], off_m[3], off_r[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int p = h + a.pad_h - r;
        const bool rok = tv && (unsigned)p < (unsigned)a.P;
        const int base = (n * a.K * a.P + p) * a.Q + v0;          // column v0 of dy (pad_w = 1: q = v)
        off_m[r] = rok ? (uint32_t)base * 4u : 0x80000000u;
        off_l[r] = (rok && v0 > 0) ? (uint32_t)(base - 1) * 4u : 0x80000000u;
        off_r[r] = (rok && v0 + 4 < a.Q) ? (uint32_t)(base + 4) * 4u : 0x80000000u;
    }

    float acc[C][4];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[c][j] = 0.f;

    for (int k = 0; k < a.K; ++k) {
        const float *wk = a.w + (int64_t)k * C * 9;        // uniform address: scalar loads
        const int so = k * PQ * 4;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // d[0..5] = dy[q = v0-1 .. v0+4] of row p
            float d[6];
            d[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off_l[r], so, 0));
            const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs, off_m[r], so, 0));
            d[5] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off_r[r], so, 0));
            d[1] = m[0]; d[2] = m[1]; d[3] = m[2]; d[4] = m[3];
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const float wv = wk[c * 9 + r * 3 + s];
                    // pixel v0+j reads q = v0 + j + 1 - s  ->  d[j + 2 - s]
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[c][j] = __builtin_fmaf(d[j + 2 - s], wv, acc[c][j]);
                }
        }
    }
    if (!tv) return;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        floatx4 o = {acc[c][0], acc[c][1], acc[c][2], acc[c][3]};
        *reinterpret_cast<floatx4 *>(a.dx + (((int64_t)n * C + c) * a.H + h) * a.W + v0) = o;
    }
}

hipError_t launch_bwd_data_smallc(const SmallCArgs &a, hipStream_t s)
{
    const int64_t total = (int64_t)a.N * a.H * (a.W >> 2);
    const dim3 grid((unsigned)((total + 255) / 256));
    switch (a.C) {
    case 1: hipLaunchKernelGGL(bwd_data_smallc_kernel<1>, grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(bwd_data_smallc_kernel<2>, grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL(bwd_data_smallc_kernel<3>, grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(bwd_data_smallc_kernel<4>, grid, dim3(256), 0, s, a); break;
    }
    return hipGetLastError();
}

}  // namespace mi355conv
