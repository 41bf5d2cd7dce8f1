// Backward-data of a first layer: 3x3, stride 1, very few input channels (C <= 4).
//
// With C = 3 the GEMM form of backward-data has only 3 useful rows out of a
// 32-row MFMA tile, so the matrix pipe cannot be used sensibly; the layer is
// bound by reading dy once (Sec. 4.1 of the paper times such layers as part of
// the convolution stack although frameworks usually skip this gradient).  This
// kernel computes it directly on the vector ALU:
//   dx[n,c,h,v] = sum_{k,r,s} dy[n,k,h+pad_h-r,v+1-s] * w[k,c,r,s]
// Each thread owns 4 consecutive pixels of one row for all C channels.  Per
// (k, r) it needs 6 values of dy: its own aligned 16 bytes (one buffer load whose
// per-thread offset is fixed; k advances through the scalar offset; rows outside
// the image carry an offset beyond the buffer and read as 0) and the pixels left
// and right of them, which are the neighbouring lanes' values and come over by
// lane shuffles (the two lanes at the ends of a wave get theirs by scalar loads).
// It then does 12*C multiply-adds whose weight operand is a scalar register (the
// weights of one k are 9*C consecutive floats of w, fetched with scalar loads).

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
    const int lane = threadIdx.x & 63;
    // fixed byte offsets inside filter plane 0 of image n: rows p = h + pad_h - r.  The pixel
    // left of a thread's four is the last one of the previous lane's four (the lanes of a wave
    // are consecutive groups of a row), the pixel to the right the first of the next lane's:
    // they come over by lane shuffles, not from memory.  Only lane 0 / lane 63 have no such
    // neighbour; theirs are wave-uniform addresses, fetched with scalar loads.
    uint32_t off_m[3];
    int edge_l[3], edge_r[3];          // element indices of the two edge pixels (wave-uniform; 0 if none)
    bool edge_lv[3], edge_rv[3];       // ... and whether they exist
    const bool has_l = v0 > 0, has_r = v0 + 4 < a.Q;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int p = h + a.pad_h - r;
        const bool rok = tv && (unsigned)p < (unsigned)a.P;
        const int base = (n * a.K * a.P + p) * a.Q + v0;          // column v0 of dy (pad_w = 1: q = v)
        off_m[r] = rok ? (uint32_t)base * 4u : 0x80000000u;
        const int el = (rok && has_l) ? base - 1 : -1, er = (rok && has_r) ? base + 4 : -1;
        const int ul = __builtin_amdgcn_readlane(el, 0), ur = __builtin_amdgcn_readlane(er, 63);
        edge_lv[r] = ul >= 0;
        edge_rv[r] = ur >= 0;
        edge_l[r] = ul >= 0 ? ul : 0;          // always an index inside the plane: the load is unconditional
        edge_r[r] = ur >= 0 ? ur : 0;
    }

    float acc[C][4];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[c][j] = 0.f;

    for (int k = 0; k < a.K; ++k) {
        const float *wk = a.w + (int64_t)k * C * 9;        // uniform address: scalar loads
        const int so = k * PQ * 4;
        const float *dyk = a.dy + (int64_t)k * PQ;         // uniform
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // d[0..5] = dy[q = v0-1 .. v0+4] of row p
            float d[6];
            const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs, off_m[r], so, 0));
            const float ld_l = dyk[edge_l[r]], ld_r = dyk[edge_r[r]];       // scalar loads
            const float wave_l = edge_lv[r] ? ld_l : 0.f;
            const float wave_r = edge_rv[r] ? ld_r : 0.f;
            // lane i <- lane i-1 and lane i <- lane i+1 through the LDS crossbar (no memory
            // access); the edge lanes take the scalar value
            const float ul = __shfl_up(m[3], 1), ur = __shfl_down(m[0], 1);
            const float sl = lane == 0 ? wave_l : ul;
            const float sr = lane == 63 ? wave_r : ur;
            d[0] = has_l ? sl : 0.f;
            d[5] = has_r ? sr : 0.f;
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
    const ProfScope ps(KID_SMALLC, 18.0 * a.N * (double)a.K * a.P * a.Q * a.C,
                       (double)a.dy_bytes + 4.0 * a.N * (double)a.C * a.H * a.W, s);
    switch (a.C) {
    case 1: hipLaunchKernelGGL(bwd_data_smallc_kernel<1>, grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(bwd_data_smallc_kernel<2>, grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL(bwd_data_smallc_kernel<3>, grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(bwd_data_smallc_kernel<4>, grid, dim3(256), 0, s, a); break;
    }
    return hipGetLastError();
}

}  // namespace mi355conv
