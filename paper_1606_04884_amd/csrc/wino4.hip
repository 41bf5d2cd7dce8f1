// Winograd F(4x4,3x3) for 3x3 stride-1 layers with many channels on small maps, with the
// transforms as separate kernels around 36 batched GEMMs on fp32 MFMA.
//
// Sec. 4.2 "Winograd" of the paper: minimal filtering trades multiplications for
// transforms, and the bulk of the work remains matrix products.  The larger tile does 36
// multiplications per 4x4 outputs and channel pair (k, c) against 144 direct ones (4x fewer;
// F(2x2,3x3) saves 2.25x).  Its 36 positions do not fit the accumulator registers of a
// fused kernel, so here the transformed tensors go through HBM:
//
//   U[pos] = G g G^T            (filters,   wino4_filter_kernel)
//   V[pos] = B^T d B            (6x6 input tiles, wino4_input_kernel)
//   M[pos] = U[pos]^T V[pos]    (36 GEMMs [K x C] . [C x tiles], wino4_gemm_kernel)
//   Y      = A^T M A + bias     (4x4 output tiles, wino4_output_kernel)
//
// which costs 2.25x the layer's input and output in extra writes and reads: small next to
// the GEMMs when C and K are in the hundreds, too much for the 64/128-channel layers on
// large maps (those stay with the fused F(2x2,3x3) kernels).  The paper prints no
// matrices; the standard ones for the points {0, 1, -1, 2, -2, inf} are used:
//   B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1]
//   G   = [1/4 0 0; -1/6 -1/6 -1/6; -1/6 1/6 -1/6; 1/24 1/12 1/6; 1/24 -1/12 1/6; 0 0 1]
//   A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
//
// Operand layout of the GEMMs ("MFMA order"): a matrix X[depth][row] is stored as
// [depth/8][depth%2][row][(depth%8)/2], so that the four values a lane of
// v_mfma_f32_32x32x2_f32 supplies for the four reduction steps of an 8-deep chunk
// (lane l: row l%32, depth 8*chunk + 2*step + l/32) are 16 contiguous bytes and the 32
// lanes of a half-wave read 512 contiguous bytes.  Both transforms write this layout, so
// the GEMM loads its operands from L2 / HBM straight into the registers the MFMAs read:
// no LDS, no barrier, waves drift freely.

#include "conv_internal.h"

#include <mutex>

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ filters
// U[pos][chunk][half][ko][j]: output channel ko < Kpad, reduction channel
// ci = 8*(chunk % csub) + 2*j + half of sub-filter q = chunk / csub (csub = chunks per
// sub-filter); zero where ci >= Cin or ko >= Kout.  A filter larger than 3x3 is the sum of
// its 3x3 sub-filters q = (a, b), taps (3a + r, 3b + s), zero where the R x S filter ends,
// applied to the input shifted by (3a, 3b); R = S = 3: one sub-filter, the filter itself.
// mode 0: g = w[ko][ci]; mode 1 (backward-data: the layer mapping dy to dx): g = w[ci][ko]
// rotated by 180 degrees.
__global__ __launch_bounds__(256) void wino4_filter_kernel(const float *__restrict__ w, float *__restrict__ U,
                                                           int C, int Cin, int Kout, int chunks, int Kpad, int mode,
                                                           int R, int S, int csub)
{
    const int nsw = (S + 2) / 3, RS = R * S;
    const int64_t nvec = (int64_t)chunks * 2 * Kpad;           // 16-byte vectors per position
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * blockDim.x) {
        const int ko = (int)(v % Kpad);
        const int ch = (int)(v / Kpad);                         // chunk * 2 + half
        floatx4 u[36];
        const int q = (ch >> 1) / csub, cchunk = (ch >> 1) - q * csub;
        const int r0 = 3 * (q / nsw), s0 = 3 * (q - (q / nsw) * nsw);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ci = cchunk * 8 + (ch & 1) + 2 * j;
            float g[3][3];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) g[r][s] = 0.f;
            if (ci < Cin && ko < Kout) {
                const float *p = mode == 0 ? w + ((int64_t)ko * C + ci) * RS : w + ((int64_t)ci * C + ko) * RS;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s) {
                        const int rr = r0 + r, ss = s0 + s;
                        if (rr < R && ss < S) g[r][s] = mode == 0 ? p[rr * S + ss] : p[(R - 1 - rr) * S + (S - 1 - ss)];
                    }
            }
            float t[6][3];
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const float g0 = g[0][s], g1 = g[1][s], g2 = g[2][s];
                t[0][s] = 0.25f * g0;
                t[1][s] = (-1.f / 6.f) * (g0 + g1 + g2);
                t[2][s] = (-1.f / 6.f) * (g0 - g1 + g2);
                t[3][s] = (1.f / 24.f) * g0 + (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
                t[4][s] = (1.f / 24.f) * g0 - (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
                t[5][s] = g2;
            }
#pragma unroll
            for (int r = 0; r < 6; ++r) {
                const float g0 = t[r][0], g1 = t[r][1], g2 = t[r][2];
                u[6 * r + 0][j] = 0.25f * g0;
                u[6 * r + 1][j] = (-1.f / 6.f) * (g0 + g1 + g2);
                u[6 * r + 2][j] = (-1.f / 6.f) * (g0 - g1 + g2);
                u[6 * r + 3][j] = (1.f / 24.f) * g0 + (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
                u[6 * r + 4][j] = (1.f / 24.f) * g0 - (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
                u[6 * r + 5][j] = g2;
            }
        }
#pragma unroll
        for (int pos = 0; pos < 36; ++pos)
            *reinterpret_cast<floatx4 *>(U + ((int64_t)pos * nvec + v) * 4) = u[pos];
    }
}

// B^T d on six values (one column, or one row, of the tile)
__device__ __forceinline__ void w4_bt(const float d0, const float d1, const float d2, const float d3,
                                      const float d4, const float d5, float (&o)[6])
{
    const float a = d4 - 4.f * d2, b = d3 - 4.f * d1;
    const float c = d4 - d2, e = 2.f * (d3 - d1);
    o[0] = 4.f * d0 - 5.f * d2 + d4;
    o[1] = a + b;
    o[2] = a - b;
    o[3] = c + e;
    o[4] = c - e;
    o[5] = 4.f * d1 - 5.f * d3 + d5;
}

// Six consecutive floats of a patch row as dword + 16 bytes + dword (buffer loads work at any
// 4-byte-aligned offset and range-check every component on its own).  `off` is the byte
// offset of the row's first element, or 0x80000000 for a row outside the image (all zeros);
// bit jj of `colbad` marks a column outside the image row: the end dwords then carry an
// out-of-range offset, the middle components are replaced by 0 (they may have read the
// neighbouring row).  Needs pad_w <= 1, so that the 16 bytes start inside the row.
__device__ __forceinline__ void w4_load_row6(const __amdgpu_buffer_rsrc_t rs, uint32_t off, int so, uint32_t colbad,
                                             float (&d)[6])
{
    const uint32_t o0 = (colbad & 1u) ? 0x80000000u : off;
    const uint32_t o5 = (colbad & 32u) ? 0x80000000u : off + 20u;
    d[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, o0, so, 0));
    const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 4u, so, 0));
    d[5] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, o5, so, 0));
    d[1] = (colbad & 2u) ? 0.f : m[0];
    d[2] = (colbad & 4u) ? 0.f : m[1];
    d[3] = (colbad & 8u) ? 0.f : m[2];
    d[4] = (colbad & 16u) ? 0.f : m[3];
}

// ------------------------------------------------------------------- input
// V[pos][chunk][half][t][j], t < Tpad (tiles past T are written as zeros), channel
// ci = 8*(chunk % csub) + 2*j + half of sub-filter chunk / csub, whose patches are shifted
// by three pixels per sub-filter row / column.  A thread owns one tile and the four channels of one
// (chunk, half): it fetches their 6x6 patches (origin 4*tile - pad; elements outside the
// image carry an offset beyond the buffer, for which the buffer load returns 0),
// transforms them and stores each position as one 16-byte vector; the 64 lanes of a wave
// are consecutive tiles, so every store instruction writes 1 KB contiguously.
__global__ __launch_bounds__(256) void wino4_input_kernel(W4Args a)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int ch = blockIdx.y;                                  // chunk * 2 + half
    if (t >= a.Tpad) return;
    const bool tv = t < a.T;
    const int tl = tv ? t : 0;
    const int THW = a.TH * a.TW;
    const int n = tl / THW, rem = tl - n * THW;
    const int th = rem / a.TW, tw = rem - th * a.TW;
    // (chunk -> sub-filter q and its chunk of real channels; the block is uniform in both)
    const int q = (ch >> 1) / a.csub, cchunk = (ch >> 1) - q * a.csub;
    const int ih0 = 4 * th - a.pad_h + 3 * (q / a.nsw), iw0 = 4 * tw - a.pad_w + 3 * (q % a.nsw);
    const int HW = a.Hin * a.Win;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, a.in_bytes, 0x00020000);
    uint32_t rowoff[6];
    uint32_t colbad = 0;
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const bool ok = tv && (unsigned)(ih0 + i) < (unsigned)a.Hin;
        rowoff[i] = ok ? (uint32_t)((n * a.Cin * HW + (ih0 + i) * a.Win + iw0) * 4) : 0x80000000u;
        if (!((unsigned)(iw0 + i) < (unsigned)a.Win)) colbad |= 1u << i;
    }
    floatx4 v[36];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int ci = cchunk * 8 + (ch & 1) + 2 * j;
        const uint32_t cbad = ci < a.Cin ? 0u : 0x80000000u;
        const int so = (ci < a.Cin ? ci : 0) * HW * 4;
        float d[6][6];
        if (a.pad_w <= 1) {
#pragma unroll
            for (int i = 0; i < 6; ++i) w4_load_row6(rs, rowoff[i] | cbad, so, colbad, d[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 6; ++i)
#pragma unroll
                for (int jj = 0; jj < 6; ++jj) {
                    const uint32_t off = ((colbad >> jj) & 1u) ? 0x80000000u : (rowoff[i] + 4u * jj);
                    d[i][jj] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off | cbad, so, 0));
                }
        }
        float tcol[6][6];       // B^T d: column pass
#pragma unroll
        for (int jj = 0; jj < 6; ++jj) {
            float o[6];
            w4_bt(d[0][jj], d[1][jj], d[2][jj], d[3][jj], d[4][jj], d[5][jj], o);
#pragma unroll
            for (int i = 0; i < 6; ++i) tcol[i][jj] = o[i];
        }
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            float o[6];
            w4_bt(tcol[i][0], tcol[i][1], tcol[i][2], tcol[i][3], tcol[i][4], tcol[i][5], o);
#pragma unroll
            for (int jj = 0; jj < 6; ++jj) v[6 * i + jj][j] = o[jj];
        }
    }
    const int64_t pos_stride = (int64_t)a.chunks * 2 * a.Tpad * 4;
    float *dst = a.V + ((int64_t)ch * a.Tpad + t) * 4;
#pragma unroll
    for (int pos = 0; pos < 36; ++pos) *reinterpret_cast<floatx4 *>(dst + pos * pos_stride) = v[pos];
}

// ------------------------------------------------------------------- GEMMs
// C[b][m][n] = sum_d A[b][d][m] * B[b][d][n] for b < 36, A and B in MFMA order (see the
// head of this file), Mpad / Npad rows per half-plane, multiples of the workgroup tile, so
// no access needs a bounds check.  A wave owns 64 rows x 128 columns (2 x 4 MFMA tiles,
// 128 accumulator registers) and per 8-deep chunk issues 2 + 4 16-byte loads and 32
// MFMAs; the loads of chunk i+1 go into a second register set during the MFMAs of chunk
// i, spread over the gaps between runs of 8 MFMAs.  Four waves per workgroup as WGM x WGN
// wave tiles, two workgroups per compute unit (two waves per SIMD: the loads of one
// overlap the MFMAs of the other).  Workgroup ids are remapped so that each XCD walks a
// contiguous range of tiles in the order (position, column tile, row tile): the B tile
// column is then reused from its L2 across the row tiles, and one position's A stays there.
__device__ __forceinline__ int w4_xcd_remap(int id, int nb)
{
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = id & 7, local = id >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}

template <int WGM, int WGN, bool BATCH_INNER, int NB>
__global__ __launch_bounds__(256, 2) void wino4_gemm_kernel(W4GemmArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    constexpr int TM = 64 * WGM, TN = 128 * WGN;
    const int lb = w4_xcd_remap(blockIdx.x, gridDim.x);
    const int piece = lb / a.nsplit, split = lb - piece * a.nsplit;
    const int tile = a.tile_base + piece;
    const int tm = tile % a.tiles_m;
    const int r1 = tile / a.tiles_m;
    const int tn = r1 % a.tiles_n;
    const int pos = r1 / a.tiles_n;
    const int wm = wave % WGM, wn = wave / WGM;
    const int m0 = (tm * WGM + wm) * 64, n0 = (tn * WGN + wn) * 128;
    // this workgroup's share of the reduction
    const int c_first = (int)((int64_t)split * a.chunks / a.nsplit);
    const int c_end = (int)((int64_t)(split + 1) * a.chunks / a.nsplit);

    // BATCH_INNER = false: A[b][chunk][half][row][4], C[b][row][col] (the Winograd transforms'
    // layout).  true: A[chunk][half][b][row][4], C[row][b][col] with NB batches (the frequency-
    // domain path: what one of its transform waves touches then lies close together)
    const int a_half = BATCH_INNER ? NB * a.Mpad * 16 : a.Mpad * 16, b_half = BATCH_INNER ? NB * a.Npad * 16 : a.Npad * 16;
    const int a_chunk = 2 * a_half, b_chunk = 2 * b_half;                     // bytes per chunk
    const float *Ap = a.A + (BATCH_INNER ? (int64_t)pos * a.Mpad * 4 : (int64_t)pos * a.chunks * 2 * a.Mpad * 4);
    const float *Bp = a.B + (BATCH_INNER ? (int64_t)pos * a.Npad * 4 : (int64_t)pos * a.chunks * 2 * a.Npad * 4);
    // exactly this batch's extent: the last chunk's second half ends the buffer
    const __amdgpu_buffer_rsrc_t ars = __builtin_amdgcn_make_buffer_rsrc(
        (void *)Ap, 0, BATCH_INNER ? (a.chunks - 1) * a_chunk + a_half + a.Mpad * 16 : a.chunks * a_chunk, 0x00020000);
    const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)Bp, 0, BATCH_INNER ? (a.chunks - 1) * b_chunk + b_half + a.Npad * 16 : a.chunks * b_chunk, 0x00020000);
    const uint32_t aoff = BATCH_INNER ? (uint32_t)(lhi * a_half) + (uint32_t)(m0 + l32) * 16u : (uint32_t)(lhi * a.Mpad + m0 + l32) * 16u;
    const uint32_t boff = BATCH_INNER ? (uint32_t)(lhi * b_half) + (uint32_t)(n0 + l32) * 16u : (uint32_t)(lhi * a.Npad + n0 + l32) * 16u;

    // three register sets: the loads of chunk i+2 are issued during the MFMAs of chunk i
    floatx4 ra[3][2], rb[3][4];
    auto load_a = [&](int set, int mi, int chunk) {
        ra[set][mi] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(ars, aoff + mi * 512u, chunk * a_chunk, 0));
    };
    auto load_b = [&](int set, int ni, int chunk) {
        rb[set][ni] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(brs, boff + ni * 512u, chunk * b_chunk, 0));
    };

    floatx16 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    const int last = c_end - 1;
    load_a(0, 0, c_first); load_a(0, 1, c_first);
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) load_b(0, ni, c_first);
    {
        const int c1 = last < c_first + 1 ? last : c_first + 1;
        load_a(1, 0, c1); load_a(1, 1, c1);
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) load_b(1, ni, c1);
    }

    // one chunk: the MFMAs of register set `cur`, the loads of chunk `nc` into set `nxt`
    auto body = [&](int cur, int nxt, int nc) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) { load_a(nxt, 0, nc); }
            if (ks == 1) { load_b(nxt, 0, nc); }
            if (ks == 2) { load_b(nxt, 2, nc); }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int mi = q & 1, ni = q >> 1;
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(ra[cur][mi][ks], rb[cur][ni][ks], acc[mi][ni], 0, 0, 0);
                if (q == 3) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks == 0) { load_a(nxt, 1, nc); }
                    if (ks == 1) { load_b(nxt, 1, nc); }
                    if (ks == 2) { load_b(nxt, 3, nc); }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    auto clampc = [&](int c) { return c < last ? c : last; };
    for (int c = c_first; c < c_end; c += 3) {
        body(0, 2, clampc(c + 2));
        if (c + 1 < c_end) body(1, 0, clampc(c + 3));
        if (c + 2 < c_end) body(2, 1, clampc(c + 4));
    }

    // accumulator element v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32
    // (a split tile goes to its slot, a dense TM x TN block)
    float *Cp = a.nsplit > 1 ? a.slots + (int64_t)lb * (TM * TN) + (wm * 64 + 4 * lhi) * TN + wn * 128 + l32
                             : BATCH_INNER ? a.C + (int64_t)pos * a.Npad + (int64_t)(m0 + 4 * lhi) * NB * a.Npad + n0 + l32
                                           : a.C + (int64_t)pos * a.Mpad * a.Npad + (int64_t)(m0 + 4 * lhi) * a.Npad + n0 + l32;
    const int64_t pitch = a.nsplit > 1 ? TN : BATCH_INNER ? (int64_t)NB * a.Npad : a.Npad;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                Cp[(int64_t)(32 * mi + 8 * (v >> 2) + (v & 3)) * pitch + 32 * ni] = acc[mi][ni][v];
}

// Sum of the depth splits of the tiles that were cut (see launch_wino4): C tile j of the
// split group = slot[j*S] + slot[j*S+1] + ... in that order.  Grid (tiles, 8): block
// (j, part) adds an eighth of the tile, 16 bytes per thread and step.
template <int TM, int TN, bool BATCH_INNER, int NB>
__global__ __launch_bounds__(256) void wino4_gemm_fixup_kernel(W4GemmArgs a)
{
    const int tile = a.tile_base + blockIdx.x;
    const int tm = tile % a.tiles_m, r1 = tile / a.tiles_m;
    const int tn = r1 % a.tiles_n, pos = r1 / a.tiles_n;
    const float *src = a.slots + (int64_t)blockIdx.x * a.nsplit * (TM * TN);
    const int64_t pitch = BATCH_INNER ? (int64_t)NB * a.Npad : a.Npad;
    float *dst = a.C + (BATCH_INNER ? (int64_t)pos * a.Npad : (int64_t)pos * a.Mpad * a.Npad) + (int64_t)tm * TM * pitch + tn * TN;
    constexpr int NV = TM * TN / 4 / 8;                 // 16-byte vectors per part
    for (int iv = threadIdx.x; iv < NV; iv += 256) {
        const int e = (blockIdx.y * NV + iv) * 4;
        const int row = e / TN, col = e - row * TN;
        floatx4 r = *reinterpret_cast<const floatx4 *>(src + e);
        for (int sp = 1; sp < a.nsplit; ++sp) {
            const floatx4 q = *reinterpret_cast<const floatx4 *>(src + (int64_t)sp * (TM * TN) + e);
            r[0] += q[0]; r[1] += q[1]; r[2] += q[2]; r[3] += q[3];
        }
        *reinterpret_cast<floatx4 *>(dst + (int64_t)row * pitch + col) = r;
    }
}

// ------------------------------------------------------------------ output
// Y = A^T M A + bias for one (filter, tile) per thread: 36 coalesced dword loads of
// M[pos][k][t] (lanes = consecutive tiles), 4 rows of the 4x4 output block stored as
// 16-byte vectors when the map allows it.
__device__ __forceinline__ void w4_at(const float m0, const float m1, const float m2, const float m3,
                                      const float m4, const float m5, float (&y)[4])
{
    const float s12 = m1 + m2, d12 = m1 - m2, s34 = m3 + m4, d34 = m3 - m4;
    y[0] = m0 + s12 + s34;
    y[1] = d12 + 2.f * d34;
    y[2] = s12 + 4.f * s34;
    y[3] = d12 + 8.f * d34 + m5;
}

__global__ __launch_bounds__(256) void wino4_output_kernel(W4Args a)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int k = blockIdx.y;
    if (t >= a.T) return;
    const int THW = a.TH * a.TW;
    const int n = t / THW, rem = t - n * THW;
    const int th = rem / a.TW, tw = rem - th * a.TW;
    const int64_t pos_stride = (int64_t)a.Kpad * a.Tpad;
    const float *src = a.M + (int64_t)k * a.Tpad + t;
    float m[6][6];
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int j = 0; j < 6; ++j) m[i][j] = src[(6 * i + j) * pos_stride];
    float c[4][6];          // A^T M: column pass
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        float y[4];
        w4_at(m[0][j], m[1][j], m[2][j], m[3][j], m[4][j], m[5][j], y);
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i][j] = y[i];
    }
    const float bz = a.bias ? a.bias[k] : 0.f;
    const int oh = 4 * th, ow = 4 * tw;
    float *o = a.out + ((int64_t)n * a.Kout + k) * a.Hout * a.Wout + (int64_t)oh * a.Wout + ow;
    const bool vec = (a.Wout & 3) == 0 && (((uintptr_t)a.out) & 15) == 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float y[4];
        w4_at(c[i][0], c[i][1], c[i][2], c[i][3], c[i][4], c[i][5], y);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            y[j] += bz;
            if (a.relu) y[j] = fmaxf(y[j], 0.f);
        }
        if (oh + i < a.Hout) {
            if (vec) {
                const floatx4 y4 = {y[0], y[1], y[2], y[3]};
                *reinterpret_cast<floatx4 *>(o + (int64_t)i * a.Wout) = y4;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (ow + j < a.Wout) o[(int64_t)i * a.Wout + j] = y[j];
            }
        }
    }
}

// ---------------------------------------------------------- backward-weight
// The tile relation is bilinear in (g, d), so the filter gradient is
//   dg = G^T [ sum over tiles (A dy A^T) .* (B^T d B) ] G
// (checked exactly on the CPU): 36 GEMMs  D[pos][k][c] = sum_t W[pos][t][k] V[pos][t][c]
// whose reduction axis is the tiles of the whole batch.  The same GEMM kernel serves: both
// operands are written in MFMA order with the TILE index as the depth, rows = filters /
// channels.  K x C is only a few workgroup tiles, so every tile is cut into depth shares
// (all go to slots); the last kernel adds the shares in order and applies G^T . G.
//

// A y on four values (a column or a row of the 4x4 gradient tile)
__device__ __forceinline__ void w4_a(const float y0, const float y1, const float y2, const float y3, float (&o)[6])
{
    const float e = y0 + y2, f = y1 + y3, g = y0 + 4.f * y2, h = 2.f * y1 + 8.f * y3;
    o[0] = y0;
    o[1] = e + f;
    o[2] = e - f;
    o[3] = g + h;
    o[4] = g - h;
    o[5] = y3;
}

// Thread mapping of the two transforms: a wave takes 8 rows (channels / filters) x the 8
// tiles of one chunk, lane = row*8 + half*4 + j with tile = 8*chunk + 2*j + half, so that a
// store instruction writes, per position, two runs of 128 contiguous bytes (the [row][j]
// vectors of both halves) and a load instruction reads 8 planes x 8 neighbouring tiles.
__global__ __launch_bounds__(256) void wino4_wg_input_kernel(W4WgradArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 3, h = (lane >> 2) & 1;
    const int c = blockIdx.x * 32 + wave * 8 + (lane >> 3);       // row: sub-filter q, channel cr
    const int tc = blockIdx.y;
    if (c >= a.Cpad) return;
    const int q = c / a.C, cr = c - q * a.C;
    const int t = tc * 8 + 2 * j + h;
    const bool tv = t < a.T && q < a.nsub;
    const int tl = t < a.T ? t : 0;
    const int HW = a.H * a.W;
    const int n = (int)fast_div((uint32_t)tl, a.div_THW), rem = tl - n * (a.TH * a.TW);
    const int th = (int)fast_div((uint32_t)rem, a.div_TW), tw = rem - th * a.TW;
    const int ih0 = 4 * th - a.pad_h + 3 * (q / a.nsw), iw0 = 4 * tw - a.pad_w + 3 * (q % a.nsw);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const int cl = q < a.nsub ? cr : 0;
    uint32_t colbad = 0;
#pragma unroll
    for (int i = 0; i < 6; ++i)
        if (!((unsigned)(iw0 + i) < (unsigned)a.W)) colbad |= 1u << i;
    float d[6][6];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const bool ok = tv && (unsigned)(ih0 + i) < (unsigned)a.H;
        const uint32_t rowoff = ok ? (uint32_t)(((n * a.C + cl) * HW + (ih0 + i) * a.W + iw0) * 4) : 0x80000000u;
        if (a.pad_w <= 1) {
            w4_load_row6(rs, rowoff, 0, colbad, d[i]);
        } else {
#pragma unroll
            for (int jj = 0; jj < 6; ++jj) {
                const uint32_t off = ((colbad >> jj) & 1u) ? 0x80000000u : (rowoff + 4u * jj);
                d[i][jj] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
            }
        }
    }
    float tcol[6][6];
#pragma unroll
    for (int jj = 0; jj < 6; ++jj) {
        float o[6];
        w4_bt(d[0][jj], d[1][jj], d[2][jj], d[3][jj], d[4][jj], d[5][jj], o);
#pragma unroll
        for (int i = 0; i < 6; ++i) tcol[i][jj] = o[i];
    }
    // The 36 results of a lane go through a wave-private LDS area [pos][lane] (the four j of a
    // (row, half) are neighbouring lanes, i.e. 16 contiguous bytes) and leave as 16-byte
    // vectors: lane (ps, v) stores positions 4*g + ps of vector v = (row, half), so a store
    // instruction writes 8 runs of 128 bytes instead of 2 (dword stores held this kernel at
    // 3.6 TB/s).  LDS operations of a wave execute in order: no barrier.
    __shared__ float sm[4][36 * 64];
    float *my = sm[wave];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        float o[6];
        w4_bt(tcol[i][0], tcol[i][1], tcol[i][2], tcol[i][3], tcol[i][4], tcol[i][5], o);
#pragma unroll
        for (int jj = 0; jj < 6; ++jj) my[(6 * i + jj) * 64 + lane] = o[jj];
    }
    const int64_t pos_stride = (int64_t)a.chunks * 2 * a.Cpad * 4;
    const int ps = lane >> 4, v = lane & 15;
    const int crow = blockIdx.x * 32 + wave * 8 + (v >> 1);
    float *dst = a.Vm + ((int64_t)(tc * 2 + (v & 1)) * a.Cpad + crow) * 4;
#pragma unroll
    for (int g = 0; g < 9; ++g) {
        const floatx4 val = *reinterpret_cast<const floatx4 *>(my + (4 * g + ps) * 64 + v * 4);
        *reinterpret_cast<floatx4 *>(dst + (4 * g + ps) * pos_stride) = val;
    }
}

// W[pos][chunk][half][k][j] = (A dy_t A^T)[pos]; also each tile's gradient sum (position
// (1,1) of A dy A^T), added over the four tiles of a (chunk, half) by lane shuffles, as
// bias_part[k][chunk*2+half]
__global__ __launch_bounds__(256) void wino4_wg_dy_kernel(W4WgradArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 3, h = (lane >> 2) & 1;
    const int k = blockIdx.x * 32 + wave * 8 + (lane >> 3);
    const int tc = blockIdx.y;
    if (k >= a.Kpad) return;
    const int t = tc * 8 + 2 * j + h;
    const bool tv = t < a.T && k < a.K;
    const int tl = t < a.T ? t : 0;
    const int PQ = a.P * a.Q;
    const int n = (int)fast_div((uint32_t)tl, a.div_THW), rem = tl - n * (a.TH * a.TW);
    const int th = (int)fast_div((uint32_t)rem, a.div_TW), tw = rem - th * a.TW;
    const int oh = 4 * th, ow = 4 * tw;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.dy_bytes, 0x00020000);
    const int kl = k < a.K ? k : 0;
    float y[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool ok = tv && oh + i < a.P;
        const uint32_t rowoff = ok ? (uint32_t)(((n * a.K + kl) * PQ + (oh + i) * a.Q + ow) * 4) : 0x80000000u;
        // (16 bytes at any 4-byte-aligned offset; components past the row end are dropped)
        const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs, rowoff, 0, 0));
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) y[i][jj] = ow + jj < a.Q ? m[jj] : 0.f;
    }
    float tcol[6][4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        float o[6];
        w4_a(y[0][jj], y[1][jj], y[2][jj], y[3][jj], o);
#pragma unroll
        for (int i = 0; i < 6; ++i) tcol[i][jj] = o[i];
    }
    const int64_t pos_stride = (int64_t)a.chunks * 2 * a.Kpad * 4;
    float *dst = a.Wm + ((int64_t)(tc * 2 + h) * a.Kpad + k) * 4 + j;
    float tsum = 0.f;
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        float o[6];
        w4_a(tcol[i][0], tcol[i][1], tcol[i][2], tcol[i][3], o);
#pragma unroll
        for (int jj = 0; jj < 6; ++jj) dst[(6 * i + jj) * pos_stride] = o[jj];
        if (i == 1) tsum = o[1];
    }
    if (a.bias_part) {
        // tiles j = 0..3 of this (row, half) sit in four neighbouring lanes
        const float s1 = tsum + __shfl_xor(tsum, 1);
        const float s2 = s1 + __shfl_xor(s1, 2);
        if (j == 0 && k < a.K) a.bias_part[(int64_t)k * (a.chunks * 2) + tc * 2 + h] = s2;
    }
}

// G^T m on six values
__device__ __forceinline__ void w4_gt(const float m0, const float m1, const float m2, const float m3,
                                      const float m4, const float m5, float (&o)[3])
{
    const float s12 = m1 + m2, s34 = m3 + m4;
    o[0] = 0.25f * m0 - (1.f / 6.f) * s12 + (1.f / 24.f) * s34;
    o[1] = (1.f / 6.f) * (m2 - m1) + (1.f / 12.f) * (m3 - m4);
    o[2] = (1.f / 6.f) * (s34 - s12) + m5;
}

// dw[k][c] = scale * G^T D[.][k][c'] G (+ dw[k][c]) from the reduced products D[pos][Kpad][Cpad];
// a thread takes one filter and four consecutive rows c' = q*C + c (lanes along c'); the 3x3
// block of sub-filter q = (a, b) lands on taps (3a.., 3b..) of the R x S gradient.
__global__ __launch_bounds__(256) void wino4_wg_output_kernel(W4WgradArgs a)
{
    const int c0 = (blockIdx.x * 256 + threadIdx.x) * 4;
    const int k = blockIdx.y;
    if (c0 >= a.nsub * a.C) return;
    const int64_t pos_stride = (int64_t)a.Kpad * a.Cpad;
    const float *p = a.D + (int64_t)k * a.Cpad + c0;
    floatx4 m[6][6];
#pragma unroll
    for (int pos = 0; pos < 36; ++pos) m[pos / 6][pos % 6] = *reinterpret_cast<const floatx4 *>(p + pos * pos_stride);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (c0 + e >= a.nsub * a.C) break;
        const int q = (c0 + e) / a.C, cr = (c0 + e) - q * a.C;
        const int r0 = 3 * (q / a.nsw), s0 = 3 * (q % a.nsw);
        float tc[3][6];
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            float o[3];
            w4_gt(m[0][j][e], m[1][j][e], m[2][j][e], m[3][j][e], m[4][j][e], m[5][j][e], o);
#pragma unroll
            for (int i = 0; i < 3; ++i) tc[i][j] = o[i];
        }
        float *dst = a.dw + ((int64_t)k * a.C + cr) * (a.R * a.S);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            float o[3];
            w4_gt(tc[i][0], tc[i][1], tc[i][2], tc[i][3], tc[i][4], tc[i][5], o);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                if (r0 + i < a.R && s0 + j < a.S) {
                    float *d1 = dst + (r0 + i) * a.S + s0 + j;
                    const float g = a.scale * o[j];
                    *d1 = a.accumulate ? *d1 + g : g;
                }
            }
        }
    }
}

// db[k] = scale * sum_q bias_part[k][q] (+ db[k]), q over the chunk halves: one workgroup per
// filter (with one wave per filter a 256-filter layer was 64 workgroups of long serial loops),
// thread t adds elements t, t+256, ... in order, each wave combines its 64 sums by a fixed tree
// of lane exchanges and the four wave sums are added in order: deterministic.
__global__ __launch_bounds__(256) void wino4_wg_bias_kernel(W4WgradArgs a)
{
    __shared__ float wsum[4];
    const int k = blockIdx.x;
    const int n = a.chunks * 2;
    const float *p = a.bias_part + (int64_t)k * n;
    float sacc = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) sacc += p[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sacc += __shfl_xor(sacc, o);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = sacc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float g = a.scale * (((wsum[0] + wsum[1]) + wsum[2]) + wsum[3]);
        a.db[k] = a.accumulate ? a.db[k] + g : g;
    }
}

// ---------------------------------------------------------------- launchers
// workgroup tile: 2 x 2, 4 x 1 or 1 x 4 wave tiles of 64 rows x 128 columns; cfg 3 (the
// frequency-domain path's small products only): 2 x 1 wave tiles, a workgroup of two waves
int wino4_tile_m(int cfg) { return cfg == 0 ? 128 : cfg == 1 ? 256 : cfg == 2 ? 64 : 128; }
int wino4_tile_n(int cfg) { return cfg == 0 ? 256 : cfg == 1 ? 128 : cfg == 2 ? 512 : 128; }

void launch_w4_gemm(const W4GemmArgs &g, int cfg, unsigned grid, hipStream_t s)
{
    if (g.batch_inner) {
        if (cfg == 0) hipLaunchKernelGGL((wino4_gemm_kernel<2, 2, true, kFftFreqs>), dim3(grid), dim3(256), 0, s, g);
        else if (cfg == 1) hipLaunchKernelGGL((wino4_gemm_kernel<4, 1, true, kFftFreqs>), dim3(grid), dim3(256), 0, s, g);
        else if (cfg == 2) hipLaunchKernelGGL((wino4_gemm_kernel<1, 4, true, kFftFreqs>), dim3(grid), dim3(256), 0, s, g);
        else hipLaunchKernelGGL((wino4_gemm_kernel<2, 1, true, kFftFreqs>), dim3(grid), dim3(128), 0, s, g);
        return;
    }
    if (cfg == 0) hipLaunchKernelGGL((wino4_gemm_kernel<2, 2, false, 0>), dim3(grid), dim3(256), 0, s, g);
    else if (cfg == 1) hipLaunchKernelGGL((wino4_gemm_kernel<4, 1, false, 0>), dim3(grid), dim3(256), 0, s, g);
    else hipLaunchKernelGGL((wino4_gemm_kernel<1, 4, false, 0>), dim3(grid), dim3(256), 0, s, g);
}

void launch_w4_fixup(const W4GemmArgs &g, int cfg, unsigned tiles, hipStream_t s)
{
    if (g.batch_inner) {
        if (cfg == 0) hipLaunchKernelGGL((wino4_gemm_fixup_kernel<128, 256, true, kFftFreqs>), dim3(tiles, 8), dim3(256), 0, s, g);
        else if (cfg == 1) hipLaunchKernelGGL((wino4_gemm_fixup_kernel<256, 128, true, kFftFreqs>), dim3(tiles, 8), dim3(256), 0, s, g);
        else if (cfg == 2) hipLaunchKernelGGL((wino4_gemm_fixup_kernel<64, 512, true, kFftFreqs>), dim3(tiles, 8), dim3(256), 0, s, g);
        else hipLaunchKernelGGL((wino4_gemm_fixup_kernel<128, 128, true, kFftFreqs>), dim3(tiles, 8), dim3(256), 0, s, g);
        return;
    }
    if (cfg == 0) hipLaunchKernelGGL((wino4_gemm_fixup_kernel<128, 256, false, 0>), dim3(tiles, 8), dim3(256), 0, s, g);
    else if (cfg == 1) hipLaunchKernelGGL((wino4_gemm_fixup_kernel<256, 128, false, 0>), dim3(tiles, 8), dim3(256), 0, s, g);
    else hipLaunchKernelGGL((wino4_gemm_fixup_kernel<64, 512, false, 0>), dim3(tiles, 8), dim3(256), 0, s, g);
}

hipError_t launch_wino4(const W4Args &a, hipStream_t s)
{
    {
        int64_t blocks = ((int64_t)a.chunks * 2 * a.Kpad + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(wino4_filter_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a.w, a.U, a.C, a.Cin, a.Kout,
                           a.chunks, a.Kpad, a.mode, a.R, a.S, a.csub);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const double in_b = (double)a.in_bytes, out_b = 4.0 * a.N * (double)a.Kout * a.Hout * a.Wout;
    const double v_b = 4.0 * 36.0 * a.chunks * 8 * (double)a.Tpad, m_b = 4.0 * 36.0 * a.Kpad * (double)a.Tpad;
    const double u_b = 4.0 * 36.0 * a.chunks * 8 * (double)a.Kpad;
    const double gemm_flops = 72.0 * a.T * (double)a.Cin * a.Kout * (a.chunks / a.csub);
    hipError_t e;
    {
        const ProfScope ps(KID_WINO4_INPUT, 0.0, in_b + v_b, s);
        hipLaunchKernelGGL(wino4_input_kernel, dim3((unsigned)((a.Tpad + 255) / 256), (unsigned)(a.chunks * 2)), dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    W4GemmArgs g = {};
    g.A = a.U; g.B = a.V; g.C = a.M;
    g.chunks = a.chunks; g.Mpad = a.Kpad; g.Npad = a.Tpad;
    g.tiles_m = a.Kpad / wino4_tile_m(a.tile_cfg);
    g.tiles_n = a.Tpad / wino4_tile_n(a.tile_cfg);
    const int tiles = 36 * g.tiles_m * g.tiles_n;
    // whole rounds of the resident workgroups, one workgroup per tile ...
    const int full = a.split > 1 ? tiles - a.split_tiles : tiles;
    if (full > 0) {
        g.tile_base = 0; g.nsplit = 1;
        const ProfScope ps(KID_WINO4_GEMM, gemm_flops * full / tiles, (u_b + v_b + m_b) * full / tiles, s);
        launch_w4_gemm(g, a.tile_cfg, (unsigned)full, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // ... and the tiles of the last, partly filled round cut into equal depth shares, so that
    // they fill the compute units too; the shares are added in a fixed order afterwards
    if (full < tiles) {
        g.tile_base = full; g.nsplit = a.split; g.slots = a.slots;
        const unsigned grid = (unsigned)((tiles - full) * a.split);
        {
            const ProfScope ps(KID_WINO4_GEMM, gemm_flops * (tiles - full) / tiles, (u_b + v_b + m_b) * (tiles - full) / tiles, s);
            launch_w4_gemm(g, a.tile_cfg, grid, s);
            e = hipGetLastError();
        }
        if (e != hipSuccess) return e;
        launch_w4_fixup(g, a.tile_cfg, (unsigned)(tiles - full), s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const ProfScope ps(KID_WINO4_OUTPUT, 0.0, m_b + out_b, s);
    hipLaunchKernelGGL(wino4_output_kernel, dim3((unsigned)((a.T + 255) / 256), (unsigned)a.Kout), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_wino4_wgrad(const W4WgradArgs &a, hipStream_t s)
{
    const double vm_b = 4.0 * 36.0 * a.chunks * 8 * (double)a.Cpad, wm_b = 4.0 * 36.0 * a.chunks * 8 * (double)a.Kpad;
    hipError_t e;
    {
        const ProfScope ps(KID_WINO4_WG_INPUT, 0.0, (double)a.x_bytes + vm_b, s);
        const dim3 gx((unsigned)((a.Cpad + 31) / 32), (unsigned)a.chunks);
        hipLaunchKernelGGL(wino4_wg_input_kernel, gx, dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    {
        const ProfScope ps(KID_WINO4_WG_DY, 0.0, (double)a.dy_bytes + wm_b, s);
        const dim3 gy((unsigned)((a.Kpad + 31) / 32), (unsigned)a.chunks);
        hipLaunchKernelGGL(wino4_wg_dy_kernel, gy, dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    W4GemmArgs g = {};
    g.A = a.Wm; g.B = a.Vm; g.C = a.D; g.slots = a.slots;
    g.chunks = a.chunks; g.Mpad = a.Kpad; g.Npad = a.Cpad;
    g.tiles_m = a.Kpad / wino4_tile_m(a.tile_cfg);
    g.tiles_n = a.Cpad / wino4_tile_n(a.tile_cfg);
    g.tile_base = 0; g.nsplit = a.split;                // >= 2: every share goes to its slot
    const unsigned grid = (unsigned)(36 * g.tiles_m * g.tiles_n * a.split);
    {
        const double slot_b = 4.0 * grid * (double)wino4_tile_m(a.tile_cfg) * wino4_tile_n(a.tile_cfg);
        const ProfScope ps(KID_WINO4_GEMM, 72.0 * a.T * (double)a.C * a.K * a.nsub, vm_b + wm_b + slot_b, s);
        launch_w4_gemm(g, a.tile_cfg, grid, s);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    // the depth shares of every tile added in order into D, then the filter transform
    launch_w4_fixup(g, a.tile_cfg, (unsigned)(36 * g.tiles_m * g.tiles_n), s);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 go((unsigned)((a.nsub * a.C + 1023) / 1024), (unsigned)a.K);
    hipLaunchKernelGGL(wino4_wg_output_kernel, go, dim3(256), 0, s, a);
    e = hipGetLastError();
    if (e != hipSuccess || !a.db) return e;
    hipLaunchKernelGGL(wino4_wg_bias_kernel, dim3((unsigned)a.K), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace mi355conv
