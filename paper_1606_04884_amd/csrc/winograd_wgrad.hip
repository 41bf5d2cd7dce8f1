// Winograd backward-weight for 3x3 stride-1 layers on fp32 MFMA (gfx950).
//
// The forward tile relation  Y = A^T [ (G g G^T) .* (B^T d B) ] A  (Sec. 4.2
// "Winograd" of the paper; matrices as in winograd.hip) is bilinear in (g, d),
// so the gradient with respect to the filter is its transpose in g:
//   dg = G^T [ sum over tiles of (A dy A^T) .* (B^T d B) ] G          F(3x3,2x2)
// with dy the 2x2 output-gradient tile and d the 4x4 input tile.  At each of the
// 16 positions the sum over tiles (and over the batch: tiles enumerate all
// images) is a GEMM  M[pos] = DY'[pos] (K x T) * V[pos]^T (T x C): 2.25x fewer
// multiplications than the direct 9-tap form.
//
// One workgroup owns 64 filters x 64 channels at all 16 positions (256
// accumulator registers per lane, as in the forward kernel) and a contiguous
// range of tiles; per step of 8 tiles both operands are loaded from NCHW with
// buffer loads (out-of-image elements: offset beyond the buffer -> hardware
// returns 0), transformed in registers and written to LDS.  The output
// transform G^T M G happens in registers; the 3x3 partial gradients go to
// part[split][K][C][9] and the ordinary split reduction adds them up
// (deterministic order).

#include "conv_internal.h"

#include <mutex>

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void lds_barrier_ww()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ int xcd_remap_ww(int id, int nb)
{
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = id & 7, local = id >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}

// LDS rows of 64 values are padded to 68 floats (68 mod 32 = 4): the 8 tiles x 4
// columns a half-wave writes then fall in 32 different banks.  Each position's
// block of 8 rows is padded to 576 floats, a multiple of 64 dwords, so that two
// positions can be written by one paired store.
constexpr int kWwKB = 64, kWwCB = 64, kWwTS = 8, kWwPitch = 68, kWwPosStride = 576;
constexpr int kWwLdsBytes = 2 * 2 * 16 * kWwPosStride * (int)sizeof(float);

__global__ __launch_bounds__(256, 1) void wino_wgrad_kernel(WinoWgradArgs a)
{
    constexpr int KB = kWwKB, CB = kWwCB, TS = kWwTS, PITCH = kWwPitch, PSTR = kWwPosStride;
    extern __shared__ float lds[];
    // As[buf][pos][tile][filter], Bs[buf][pos][tile][channel]
    float *const As = lds;
    float *const Bs = lds + 2 * 16 * PSTR;
    static_assert(TS * PITCH <= PSTR, "position block");
    auto as_at = [&](int buf, int pos, int t, int k) -> float & { return As[(buf * 16 + pos) * PSTR + t * PITCH + k]; };
    auto bs_at = [&](int buf, int pos, int t, int c) -> float & { return Bs[(buf * 16 + pos) * PSTR + t * PITCH + c]; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;

    const int ntile = a.tiles_k * a.tiles_c;
    const int logical = xcd_remap_ww(blockIdx.x, gridDim.x);
    const int tile_id = logical % ntile;
    const int split = logical / ntile;
    const int kt = tile_id % a.tiles_k;
    const int ctv = tile_id / a.tiles_k;          // channel tile over nsub * C virtual channels
    const int sq = ctv / a.tiles_c_sub;           // sub-filter group: input shifted by (dh, dw)
    const int ct = ctv - sq * a.tiles_c_sub;
    const int sub_dh = sq == 0 ? a.sub_dh[0] : sq == 1 ? a.sub_dh[1] : sq == 2 ? a.sub_dh[2] : a.sub_dh[3];
    const int sub_dw = sq == 0 ? a.sub_dw[0] : sq == 1 ? a.sub_dw[1] : sq == 2 ? a.sub_dw[2] : a.sub_dw[3];
    const int t_begin = split * a.tiles_per_split;
    const int t_end = min(a.T, t_begin + a.tiles_per_split);
    const int nsteps = (t_end - t_begin + TS - 1) / TS;

    // this thread: tile (lane % 8) of every step; channels / filters sub, sub + 32
    const int tile_l = lane & 7;
    const int sub = tid >> 3;
    const int c0 = ct * CB + sub, k0 = kt * KB + sub;
    const int HW = a.H * a.W, PQ = a.P * a.Q;
    const bool c0ok = c0 < a.C, k0ok = k0 < a.K;
    // the "+32" items exist or not for the whole workgroup (C, K multiples of 32):
    // a descriptor of size 0 makes every load of a missing item return 0
    const __amdgpu_buffer_rsrc_t xrs0 = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrs1 =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (ct * CB + 32 < a.C) ? a.x_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t drs0 = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.dy_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t drs1 =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, (kt * KB + 32 < a.K) ? a.dy_bytes : 0, 0x00020000);
    const int xs1 = 32 * HW * 4, ds1 = 32 * PQ * 4;

    uint32_t eoff[16], doff[4];
    float xr[2][16], dr[2][4];

    auto setup = [&](int step) {
        const int tile = t_begin + step * TS + tile_l;
        const bool tv = tile < t_end;
        const int tl = tv ? tile : 0;
        const int n = (int)fast_div((uint32_t)tl, a.div_THW);
        const int rem = tl - n * (a.TH * a.TW);
        const int th = (int)fast_div((uint32_t)rem, a.div_TW);
        const int tw = rem - th * a.TW;
        const int ih0 = 2 * th - a.pad_h + sub_dh, iw0 = 2 * tw - a.pad_w + sub_dw;
        const int xbase = ((n * a.C + c0) * a.H + ih0) * a.W + iw0;
        bool rok[4], cok[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            rok[i] = tv && c0ok && (unsigned)(ih0 + i) < (unsigned)a.H;
            cok[i] = (unsigned)(iw0 + i) < (unsigned)a.W;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                eoff[4 * i + j] = (rok[i] && cok[j]) ? (uint32_t)(xbase + i * a.W + j) * 4u : 0x80000000u;
        const int dbase = ((n * a.K + k0) * a.P + 2 * th) * a.Q + 2 * tw;
        const bool r1 = 2 * th + 1 < a.P, q1 = 2 * tw + 1 < a.Q, dv = tv && k0ok;
        doff[0] = dv ? (uint32_t)dbase * 4u : 0x80000000u;
        doff[1] = (dv && q1) ? (uint32_t)(dbase + 1) * 4u : 0x80000000u;
        doff[2] = (dv && r1) ? (uint32_t)(dbase + a.Q) * 4u : 0x80000000u;
        doff[3] = (dv && r1 && q1) ? (uint32_t)(dbase + a.Q + 1) * 4u : 0x80000000u;
    };
    auto load_x = [&](int it, int e) {
        xr[it][e] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(it ? xrs1 : xrs0, eoff[e], it ? xs1 : 0, 0));
    };
    auto load_d = [&](int it, int e) {
        dr[it][e] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(it ? drs1 : drs0, doff[e], it ? ds1 : 0, 0));
    };

    // input transform V = B^T d B of item `it`: four column pieces, four row pieces
    float tr[2][16];
    auto xform_col = [&](int it, int j) {
        const float d0 = xr[it][0 + j], d1 = xr[it][4 + j], d2 = xr[it][8 + j], d3 = xr[it][12 + j];
        tr[it][0 + j] = d0 - d2;
        tr[it][4 + j] = d1 + d2;
        tr[it][8 + j] = d2 - d1;
        tr[it][12 + j] = d1 - d3;
    };
    auto xform_row_store = [&](int buf, int it, int i) {
        const float t0 = tr[it][4 * i + 0], t1 = tr[it][4 * i + 1], t2 = tr[it][4 * i + 2], t3 = tr[it][4 * i + 3];
        const int c = sub + 32 * it;
        bs_at(buf, 4 * i + 0, tile_l, c) = t0 - t2;
        bs_at(buf, 4 * i + 1, tile_l, c) = t1 + t2;
        bs_at(buf, 4 * i + 2, tile_l, c) = t2 - t1;
        bs_at(buf, 4 * i + 3, tile_l, c) = t1 - t3;
    };
    // gradient-tile transform DY' = A dy A^T, A = [1 0; 1 1; 1 -1; 0 -1]; piece i = row i
    float bsum[2] = {0.f, 0.f};      // running sum of this thread's gradient tiles (bias gradient)
    auto dyform_row_store = [&](int buf, int it, int i) {
        const float y00 = dr[it][0], y01 = dr[it][1], y10 = dr[it][2], y11 = dr[it][3];
        if (i == 0) bsum[it] += (y00 + y01) + (y10 + y11);
        float t0, t1;       // row i of A dy
        if (i == 0) { t0 = y00; t1 = y01; }
        else if (i == 1) { t0 = y00 + y10; t1 = y01 + y11; }
        else if (i == 2) { t0 = y00 - y10; t1 = y01 - y11; }
        else { t0 = -y10; t1 = -y11; }
        const int k = sub + 32 * it;
        as_at(buf, 4 * i + 0, tile_l, k) = t0;
        as_at(buf, 4 * i + 1, tile_l, k) = t0 + t1;
        as_at(buf, 4 * i + 2, tile_l, k) = t0 - t1;
        as_at(buf, 4 * i + 3, tile_l, k) = -t1;
    };

    floatx16 acc[16];
#pragma unroll
    for (int p = 0; p < 16; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;

    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    float ao[2][2][4], bo[2][2][4];
    auto read_pair = [&](int buf, int pair, int set) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                ao[set][u][ks] = as_at(buf, 2 * pair + u, 2 * ks + lhi, wm0 + l32);
                bo[set][u][ks] = bs_at(buf, 2 * pair + u, 2 * ks + lhi, wn0 + l32);
            }
    };
    auto load_all = [&]() {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
#pragma unroll
            for (int e = 0; e < 16; ++e) load_x(it, e);
#pragma unroll
            for (int e = 0; e < 4; ++e) load_d(it, e);
        }
    };

    // ---- prologue: step 0 into LDS buffer 0, step 1 into registers ----
    setup(0);
    load_all();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) xform_col(it, j);
#pragma unroll
        for (int i = 0; i < 4; ++i) xform_row_store(0, it, i);
#pragma unroll
        for (int i = 0; i < 4; ++i) dyform_row_store(0, it, i);
    }
    setup(1);            // steps past the end: every offset out of range, all zeros
    load_all();
    lds_barrier_ww();
    read_pair(0, 0, 0);

    // Software pipeline, as in the forward kernel: 64 MFMA slots per step.
    //   slots  0..15 : input transform + LDS writes of step t+1 (two items)
    //   slots 16..23 : gradient-tile transform + LDS writes of step t+1
    //   slot   1     : tile coordinates and buffer offsets of step t+2
    //   slots  4..43 : the 40 buffer loads of step t+2, each register reloaded as
    //                  soon as the transform has consumed it, so that every load
    //                  has at least 36 slots until its value is needed
    for (int t = 0; t < nsteps; ++t) {
        const int buf = t & 1;
#pragma unroll
        for (int pair = 0; pair < 8; ++pair) {
            const int cur = pair & 1, nxt = cur ^ 1;
            if (pair + 1 < 8) {
                read_pair(buf, pair + 1, nxt);
            } else {
                lds_barrier_ww();
                read_pair(buf ^ 1, 0, nxt);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int s = pair * 8 + q;
                if (s < 16) {
                    const int it = s >> 3, piece = s & 7;
                    if (piece < 4) xform_col(it, piece); else xform_row_store(buf ^ 1, it, piece - 4);
                } else if (s < 24) {
                    const int it = (s - 16) >> 2, i = (s - 16) & 3;
                    dyform_row_store(buf ^ 1, it, i);
                }
                if (s == 1) setup(t + 2);
                if (s >= 4 && s < 44) {
                    // in consumption order: x item 0 (column major), x item 1, gradient tiles
                    const int l = s - 4;
                    if (l < 32) {
                        const int it = l >> 4, j = (l >> 2) & 3, i = l & 3;
                        load_x(it, 4 * i + j);
                    } else {
                        load_d((l - 32) >> 2, (l - 32) & 3);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                const int u = q & 1, ks = q >> 1;
                acc[2 * pair + u] = __builtin_amdgcn_mfma_f32_32x32x2f32(ao[cur][u][ks], bo[cur][u][ks],
                                                                          acc[2 * pair + u], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- bias gradient: every tile of the range went through bsum exactly once.
    // Only the workgroups of channel tile 0 write it: one partial per (split, k).
    if (a.bias_part != nullptr && ctv == 0) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            float v = bsum[it];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            const int k = k0 + 32 * it;
            if (tile_l == 0 && k < a.K) a.bias_part[split * a.K + k] = v;
        }
    }

    // ---- epilogue: dg = G^T M G in registers, partial 3x3 gradients out ----
    const int c = ct * CB + wn0 + l32;
    if (c >= a.C) return;
    const int Cv = a.nsub * a.C;                  // columns of a partial matrix
    float *out = a.part + (int64_t)split * a.K * Cv * 9 + (int64_t)sq * a.C * 9;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int k = kt * KB + wm0 + 8 * (v >> 2) + 4 * lhi + (v & 3);
        if (k >= a.K) continue;
        float tt[3][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m0 = acc[0 + j][v], m1 = acc[4 + j][v], m2 = acc[8 + j][v], m3 = acc[12 + j][v];
            const float hs = 0.5f * (m1 + m2), hd = 0.5f * (m1 - m2);
            tt[0][j] = m0 + hs;
            tt[1][j] = hd;
            tt[2][j] = hs + m3;
        }
        float *o = out + ((int64_t)k * Cv + c) * 9;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const float hs = 0.5f * (tt[r][1] + tt[r][2]), hd = 0.5f * (tt[r][1] - tt[r][2]);
            o[3 * r + 0] = tt[r][0] + hs;
            o[3 * r + 1] = hd;
            o[3 * r + 2] = hs + tt[r][3];
        }
    }
}

// ---------------------------------------------------------------------------
// Vector-load variant for pad_w = 1 and even image width (then Q = W).
//
// A thread owns one channel (and one filter) and a PAIR of horizontally adjacent
// tiles per step: the two 4x4 patches overlap in two columns, so the pair is a
// 4 x 6 block fetched per row as dword + 16 bytes + dword (the 16 bytes start at
// an even column: always inside the row), the two gradient tiles are one
// 16-byte load per row, the column half of B^T d B is shared by the two
// patches, and both tiles' values of a position go out in one paired LDS store.
// The tile grid is taken with its width
// rounded up to even so that a pair never straddles two tile rows; when the true
// width is odd (ODD) the last pair of a row has a phantom right tile: its
// gradient tile and the image columns past the edge are fetched with 8-byte
// loads of their own whose offset is out of range, so they read as zero and
// the phantom contributes nothing.
//
// LDS operand planes are [buf][pos][half][64 columns][4]: the four reduction
// steps (tiles 2*ks + half, ks = 0..3) of a column are 16 contiguous bytes, so
// an MFMA operand for all four steps of a position is one 16-byte read at a
// fixed per-lane address plus an immediate.  Signs: the rows/columns of
// A dy A^T that carry a minus sign (index 3) are stored without it; the output
// transform subtracts instead of adds there.

template <int V> struct IntC { static constexpr int value = V; };

constexpr int kWvPlane = 512;                          // floats per (buf, pos): 2 halves x 64 x 4
constexpr int kWvOperand = 2 * 16 * kWvPlane;          // floats per operand (two buffers)
constexpr int kWvLdsBytes = 2 * kWvOperand * (int)sizeof(float);

// Eight waves, two per SIMD, so that the loads, LDS traffic and barrier waits of one
// wave fall under the other wave's MFMAs.  Waves 4*PH .. 4*PH+3 keep the 8 positions
// 8*PH .. 8*PH+7 (rows 2*PH, 2*PH+1 of the 4x4 position grid) of the four 32x32
// quadrants; thread (PH, channel, pair) produces exactly those rows of B^T d B and
// |A| dy |A|^T for its channel / filter and tile pair, for which it needs 3 of the 4
// patch rows (PH .. PH+2) and both gradient rows: 11 loads per step and thread, half
// the transform and LDS-store work of a thread that did all 16 positions.  At the end
// the waves of PH = 1 hand their accumulators to PH = 0 through LDS (the operand
// buffers, free by then), which applies the output transform.
// ---------------------------------------------------------------------------
template <bool ODD, int PH>
__device__ __forceinline__ void wino_wgrad_vec_body(const WinoWgradArgs &a, float *lds)
{
    constexpr int KB = kWwKB, CB = kWwCB, TS = kWwTS;
    constexpr int NXO = ODD ? 4 : 3, NDO = ODD ? 2 : 1;
    float *const As = lds;
    float *const Bs = lds + kWvOperand;

    const int tid = threadIdx.x & 255;               // index inside the PH group
    const int lane = tid & 63;
    const int wq = __builtin_amdgcn_readfirstlane(tid >> 6);      // quadrant
    const int l32 = lane & 31, lhi = lane >> 5;

    const int ntile = a.tiles_k * a.tiles_c;
    const int logical = xcd_remap_ww(blockIdx.x, gridDim.x);
    const int tile_id = logical % ntile;
    const int split = logical / ntile;
    const int kt = tile_id % a.tiles_k;
    const int ct = tile_id / a.tiles_k;
    const int t_begin = split * a.tiles_per_split;
    const int t_end = min(a.T, t_begin + a.tiles_per_split);
    const int nsteps = (t_end - t_begin + TS - 1) / TS;

    const int pr = tid & 3, ch = tid >> 2;           // tile pair of the step, channel / filter
    const int c = ct * CB + ch, k = kt * KB + ch;
    const bool cok = c < a.C, kok = k < a.K;
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t drs = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.dy_bytes, 0x00020000);

    uint32_t xo[3][NXO], dof[2][NDO];                // patch rows PH .. PH+2, gradient rows 0, 1
    float xr[3][6], dr[2][4];

    auto setup = [&](int step) {
        const int tb = t_begin + step * TS + 2 * pr;
        const bool tv = tb < t_end;
        const int tl = tv ? tb : 0;
        const int n = (int)fast_div((uint32_t)tl, a.div_THW);
        const int rem = tl - n * (a.TH * a.TW);
        const int th = (int)fast_div((uint32_t)rem, a.div_TW);
        const int tw = rem - th * a.TW;                 // even
        const int ih0 = 2 * th - a.pad_h + PH, col0 = 2 * tw;
        const int xbase = ((n * a.C + c) * a.H + ih0) * a.W + col0;
        const bool lok = tw > 0, hok = col0 + 3 < a.W, rgt = col0 + 4 < a.W;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const bool rok = tv && cok && (unsigned)(ih0 + i) < (unsigned)a.H;
            const uint32_t m = (uint32_t)(xbase + i * a.W) * 4u;
            xo[i][0] = (rok && lok) ? m - 4u : 0x80000000u;
            xo[i][1] = rok ? m : 0x80000000u;
            if (ODD) xo[i][2] = (rok && hok) ? m + 8u : 0x80000000u;
            xo[i][NXO - 1] = (rok && rgt) ? m + 16u : 0x80000000u;
        }
        const int dbase = ((n * a.K + k) * a.P + 2 * th) * a.Q + col0;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const bool dok = tv && kok && 2 * th + r < a.P;
            const uint32_t m = (uint32_t)(dbase + r * a.Q) * 4u;
            dof[r][0] = dok ? m : 0x80000000u;
            if (ODD) dof[r][1] = (dok && hok) ? m + 8u : 0x80000000u;
        }
    };
    auto load_x = [&](int i, int part) {
        if (part == 0) {
            xr[i][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrs, xo[i][0], 0, 0));
        } else if (part == NXO - 1) {
            xr[i][5] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrs, xo[i][NXO - 1], 0, 0));
        } else if (!ODD) {
            const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(xrs, xo[i][1], 0, 0));
            xr[i][1] = m[0]; xr[i][2] = m[1]; xr[i][3] = m[2]; xr[i][4] = m[3];
        } else {
            const floatx2 m = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(xrs, xo[i][part], 0, 0));
            xr[i][2 * part - 1] = m[0]; xr[i][2 * part] = m[1];
        }
    };
    auto load_d = [&](int r, int part) {
        if (!ODD) {
            const floatx4 m = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(drs, dof[r][0], 0, 0));
            dr[r][0] = m[0]; dr[r][1] = m[1]; dr[r][2] = m[2]; dr[r][3] = m[3];
        } else {
            const floatx2 m = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(drs, dof[r][part], 0, 0));
            dr[r][2 * part] = m[0]; dr[r][2 * part + 1] = m[1];
        }
    };
    constexpr int NXL = 3 * NXO;                      // image loads per step
    constexpr int NLOAD = NXL + 2 * NDO;
    auto load_nth = [&](int l) {
        if (l < NXL) load_x(l / NXO, l % NXO); else load_d((l - NXL) / NDO, (l - NXL) % NDO);
    };

    const int wofs = ch * 4 + pr;
    float tc[2][6];                                   // rows 2*PH, 2*PH+1 of B^T d
    auto xform_col = [&](int j) {
        // xr[0..2] = patch rows PH .. PH+2
        if (PH == 0) {
            tc[0][j] = xr[0][j] - xr[2][j];           // d0 - d2
            tc[1][j] = xr[1][j] + xr[2][j];           // d1 + d2
        } else {
            tc[0][j] = xr[1][j] - xr[0][j];           // d2 - d1
            tc[1][j] = xr[0][j] - xr[2][j];           // d1 - d3
        }
    };
    auto xform_row_store = [&](int buf, int il, int h) {
        const float t0 = tc[il][2 * h + 0], t1 = tc[il][2 * h + 1], t2 = tc[il][2 * h + 2], t3 = tc[il][2 * h + 3];
        float *o = Bs + (buf * 16 + 4 * (2 * PH + il)) * kWvPlane + h * 256 + wofs;
        o[0 * kWvPlane] = t0 - t2;
        o[1 * kWvPlane] = t1 + t2;
        o[2 * kWvPlane] = t2 - t1;
        o[3 * kWvPlane] = t1 - t3;
    };
    float bsum = 0.f;
    auto dyform_row_store = [&](int buf, int il, int h) {
        const float y00 = dr[0][2 * h], y01 = dr[0][2 * h + 1], y10 = dr[1][2 * h], y11 = dr[1][2 * h + 1];
        const int i = 2 * PH + il;
        float t0, t1;       // row i of |A| dy (row 3 without its sign)
        if (i == 0) { t0 = y00; t1 = y01; }
        else if (i == 1) { t0 = y00 + y10; t1 = y01 + y11; }
        else if (i == 2) { t0 = y00 - y10; t1 = y01 - y11; }
        else { t0 = y10; t1 = y11; }
        const float sum = t0 + t1;
        if (i == 1) bsum += sum;                       // all four values of the tile
        float *o = As + (buf * 16 + 4 * i) * kWvPlane + h * 256 + wofs;
        o[0 * kWvPlane] = t0;
        o[1 * kWvPlane] = sum;
        o[2 * kWvPlane] = t0 - t1;
        o[3 * kWvPlane] = t1;                          // column 3 without its sign
    };

    floatx16 acc[8];                                  // positions 8*PH + p
#pragma unroll
    for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;

    const int wm0 = (wq >> 1) * 32, wn0 = (wq & 1) * 32;
    const float *const rdA = As + (8 * PH) * kWvPlane + lhi * 256 + (wm0 + l32) * 4;
    const float *const rdB = Bs + (8 * PH) * kWvPlane + lhi * 256 + (wn0 + l32) * 4;
    floatx4 ao[2][2], bo[2][2];
    auto read_pair = [&](int buf, int pair, int set) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            ao[set][u] = *reinterpret_cast<const floatx4 *>(rdA + (buf * 16 + 2 * pair + u) * kWvPlane);
            bo[set][u] = *reinterpret_cast<const floatx4 *>(rdB + (buf * 16 + 2 * pair + u) * kWvPlane);
        }
    };

    // ---- prologue: step 0 into LDS buffer 0, step 1 into registers ----
    setup(0);
#pragma unroll
    for (int l = 0; l < NLOAD; ++l) load_nth(l);
#pragma unroll
    for (int j = 0; j < 6; ++j) xform_col(j);
#pragma unroll
    for (int q = 0; q < 4; ++q) { xform_row_store(0, q >> 1, q & 1); dyform_row_store(0, q >> 1, q & 1); }
    setup(1);            // steps past the end: every offset out of range, all zeros
#pragma unroll
    for (int l = 0; l < NLOAD; ++l) load_nth(l);
    setup(2);
    lds_barrier_ww();
    read_pair(0, 0, 0);

    // A step of a wave is 4 groups of 8 back-to-back MFMAs (two positions x four
    // reduction steps).  Gaps before the groups:
    //   gap 0 : column half of the input transform of step t+1, first image load of t+2
    //   gap 1 : row half + LDS stores (one piece per row and tile), an image load of step
    //           t+2 after every piece
    //   gap 2 : gradient-tile pieces + LDS stores, the remaining image loads
    //   gap 3 : gradient loads of step t+2, coordinates of step t+3, barrier, first
    //           operands of the next step
    // (the image loads after the first are spread as evenly as they go over the 8 pieces)
    constexpr int XREST = NXL - 1;                    // image loads after the first
    auto step_body = [&](int t, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int pair = 0; pair < 4; ++pair) {
            const int cur = pair & 1, nxt = cur ^ 1;
            if (pair + 1 < 4) {
                read_pair(buf, pair + 1, nxt);
            } else {
                lds_barrier_ww();
                read_pair(buf ^ 1, 0, nxt);
            }
            if (pair == 0) {
#pragma unroll
                for (int j = 0; j < 6; ++j) xform_col(j);
                __builtin_amdgcn_sched_barrier(0);
                load_nth(0);
            } else if (pair == 1 || pair == 2) {
#pragma unroll
                for (int q = 4 * (pair - 1); q < 4 * pair; ++q) {
                    if (pair == 1) xform_row_store(buf ^ 1, q >> 1, q & 1);
                    else dyform_row_store(buf ^ 1, (q - 4) >> 1, q & 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int l = 1 + q * XREST / 8; l < 1 + (q + 1) * XREST / 8; ++l) {
                        load_nth(l);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
#pragma unroll
                for (int l = NXL; l < NLOAD; ++l) {
                    load_nth(l);
                    __builtin_amdgcn_sched_barrier(0);
                }
                setup(t + 3);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int u = q & 1, ks = q >> 1;
                acc[2 * pair + u] = __builtin_amdgcn_mfma_f32_32x32x2f32(ao[cur][u][ks], bo[cur][u][ks],
                                                                          acc[2 * pair + u], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // an odd step count runs one extra all-zero step
    for (int t = 0; t < nsteps; t += 2) {
        step_body(t, IntC<0>());
        step_body(t + 1, IntC<1>());
    }

    // ---- bias gradient: every tile of the range went through bsum exactly once (PH 0) ----
    if (PH == 0 && a.bias_part != nullptr && ct == 0) {
        float v = bsum;
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        if (pr == 0 && kok) a.bias_part[split * a.K + k] = v;
    }

    // ---- PH 1 hands its accumulators over: [quadrant][position][v][lane] ----
    __syncthreads();                                  // every wave is done with the operand buffers
    float *const xch = lds + (wq * 8) * 16 * 64 + lane;
    if (PH == 1) {
#pragma unroll
        for (int p = 0; p < 8; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) xch[(p * 16 + v) * 64] = acc[p][v];
    }
    __syncthreads();
    if (PH == 1) return;

    // ---- epilogue: dg = G^T M G in registers (index-3 rows / columns enter with a
    // minus sign, see above), partial 3x3 gradients out ----
    const int co = ct * CB + wn0 + l32;
    if (co >= a.C) return;
    float *out = a.part + (int64_t)split * a.K * a.C * 9;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int ko = kt * KB + wm0 + 8 * (v >> 2) + 4 * lhi + (v & 3);
        if (ko >= a.K) continue;
        float tt[3][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m0 = acc[0 + j][v], m1 = acc[4 + j][v];
            const float m2 = xch[((0 + j) * 16 + v) * 64], m3 = xch[((4 + j) * 16 + v) * 64];
            const float hs = 0.5f * (m1 + m2), hd = 0.5f * (m1 - m2);
            tt[0][j] = m0 + hs;
            tt[1][j] = hd;
            tt[2][j] = hs - m3;
        }
        float *o = out + ((int64_t)ko * a.C + co) * 9;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const float hs = 0.5f * (tt[r][1] + tt[r][2]), hd = 0.5f * (tt[r][1] - tt[r][2]);
            o[3 * r + 0] = tt[r][0] + hs;
            o[3 * r + 1] = hd;
            o[3 * r + 2] = hs - tt[r][3];
        }
    }
}

template <bool ODD>
__global__ __launch_bounds__(512, 1) void wino_wgrad_vec_kernel(WinoWgradArgs a)
{
    extern __shared__ float lds[];
    // both halves run the same sequence of barriers
    if (threadIdx.x < 256) wino_wgrad_vec_body<ODD, 0>(a, lds);
    else wino_wgrad_vec_body<ODD, 1>(a, lds);
}

int wino_wgrad_tile() { return kWwKB; }
int wino_wgrad_step() { return kWwTS; }

hipError_t launch_wino_wgrad(const WinoWgradArgs &a, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t cfg = hipSuccess;
    std::call_once(once, [] {
        cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_wgrad_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kWwLdsBytes);
        if (cfg == hipSuccess)
            cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_wgrad_vec_kernel<false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kWvLdsBytes);
        if (cfg == hipSuccess)
            cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(wino_wgrad_vec_kernel<true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kWvLdsBytes);
    });
    if (cfg != hipSuccess) return cfg;
    const dim3 grid((unsigned)(a.tiles_k * a.tiles_c * a.splits));
    const ProfScope ps(a.mode == 0 ? KID_WINO_WGRAD : KID_WINO_WGRAD_VEC, 32.0 * a.T * (double)a.C * a.K * a.nsub,
                       (double)a.x_bytes + (double)a.dy_bytes + 36.0 * a.K * (double)a.C * a.nsub, s);
    if (a.mode == 0)
        hipLaunchKernelGGL(wino_wgrad_kernel, grid, dim3(256), kWwLdsBytes, s, a);
    else if (a.mode == 1)
        hipLaunchKernelGGL(wino_wgrad_vec_kernel<false>, grid, dim3(512), kWvLdsBytes, s, a);
    else
        hipLaunchKernelGGL(wino_wgrad_vec_kernel<true>, grid, dim3(512), kWvLdsBytes, s, a);
    return hipGetLastError();
}

}  // namespace mi355conv
