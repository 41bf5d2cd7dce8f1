// Pointwise (1x1, stride 1, unpadded) convolution layers for gfx950.
//
// For such a layer the lowered matrix of Sec. 4.2 of the paper is the tensor
// itself: every image is a [channels x H*W] matrix with the pixels contiguous, so
// forward, backward-data and backward-weight are plain products with it.  With
// the channel counts of an inception module (Sec. 4.1 lists GoogLeNet among the
// workloads) these products do fewer than 100 flops per byte of tensor traffic
// and are bound by HBM, not by the matrix pipe.  The kernels here are therefore
// built to stream: every tensor element is fetched from HBM exactly once, straight
// into the registers an MFMA reads (no staging of the big operand in LDS, no
// workgroup barrier in the main loop), with several KB of loads in flight per wave.
//
//   pw_stream_kernel : out[n][r][p] = bias[r] + sum_d A[r][d] * in[n][d][p]   (optionally max(0, .))
//                      (forward: A = w; backward-data: A = w transposed)
//   pw_wgrad_kernel  : part[s][k][c] = sum_{pixels of range s} dy[n][k][p] * x[n][c][p]
//
// v_mfma_f32_32x32x2_f32 operand layout (streaming kernel): lane l supplies A[i = l%32]
// [kk = l/32] and B[kk = l/32][j = l%32]; accumulator register v of lane l is row
// 8*(v/4) + 4*(l/32) + v%4, column l%32.

#include "conv_internal.h"

#include <mutex>

namespace mi355conv {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------- streaming ---
// A wave owns 32-pixel tiles (pixels = MFMA columns, lanes along the pixels: each
// B operand is one coalesced dword load of two channel rows) and all 32*MI output
// rows.  The small matrix A sits in LDS in operand order: block (g, mi) holds, for
// lane l, the four values A[32*mi + l%32][8*g + 2*e + l/32], e = 0..3, as one
// 16-byte vector, so one LDS read feeds four MFMAs.  Blocks are padded by 16 bytes
// so that the fill (consecutive depths or rows from consecutive threads) spreads
// over the banks.
constexpr int kPwBlk = 260;      // floats per block: 64 lanes x 4, + 4
constexpr int kPwRing = 8;       // 8-channel groups in flight per wave (32 loads); RING below
constexpr int kPwThreads = 512;  // eight waves share one copy of A in LDS, two per SIMD
constexpr int kPwWaves = kPwThreads / 64;
constexpr size_t kPwLdsMax = 160 * 1024;

static int pw_row_tiles(int Rout)
{
    const int t = (Rout + 31) / 32;
    if (t <= 4) return t;
    if (t <= 6) return 6;
    if (t <= 8) return 8;
    return 0;
}

size_t pw_stream_lds_bytes(int Rout, int D)
{
    const int MI = pw_row_tiles(Rout);
    if (MI == 0) return 0;
    // A blocks, bias per row, and (grouped outputs) a 16-byte destination record per row
    // (and, for the taps form, 8 bytes per depth index, padding groups of the ring included)
    const size_t bytes = ((size_t)((D + 7) / 8) * MI * kPwBlk + 32 * MI + 4 * 32 * MI + 2 * 8 * ((D + 7) / 8 + kPwRing)) * sizeof(float);
    return bytes <= kPwLdsMax ? bytes : 0;
}

// Wide stores: a wave passes each 32 x 32 block of results through a private LDS area
// (rows 40 floats apart) so that a lane ends up with four consecutive pixels of one row.
constexpr int kPwStageStride = 40;
constexpr size_t kPwStageBytes = (size_t)kPwWaves * 32 * kPwStageStride * sizeof(float);

//
// TAPS: the same kernel as the forward pass of a layer whose whole filter bank fits in LDS
// (K*C*R*S floats: first layers, the inception 5x5): the depth index d then runs over the
// taps (c, r, t) of the lowered matrix, and the dword a lane fetches for depth d is
// in[n][c][p*stride - pad_h + r][q*stride - pad_w + t] of its output pixel (p, q).  The
// element offset and (r, t) of every tap sit in an LDS table; the two half-waves read their
// two entries (a broadcast read each), and a lane tests a tap against the set of window
// rows and columns that lie inside its image, worked out once per tile.
// tap_bwd: the stride-1 backward-data pass in the same form, dx[n][c][h][u] = sum over
// (k, r, t) of w[k][c][r][t] * dy[n][k][h + pad_h - r][u + pad_w - t]: rows = c, depth =
// (k, r, t) in the filters' memory order, the window over dy starts at (h + pad_h - (R-1),
// u + pad_w - (S-1)) and tap (r, t) reads its element (R-1-r, S-1-t).
template <int MI, bool GROUPED, bool TAPS, int RING>
__global__ __launch_bounds__(kPwThreads) void pw_stream_kernel(PwArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int G8 = (a.D + 7) >> 3;
    const int Gp = (G8 + RING - 1) / RING * RING;     // see the ring below
    float *biasl = lds + G8 * MI * kPwBlk;       // [32 * MI]
    // grouped outputs: row r -> {address of its first pixel in image 0, image stride}
    struct RowDst {
        float *base;
        int32_t img_stride, unused;
    };
    RowDst *rowdst = reinterpret_cast<RowDst *>(biasl + 32 * MI);      // [32 * MI]
    // TAPS: depth d -> {byte offset of tap (c, r, t) from the window origin, 1 << r | 1 << (16 + t)}
    int2 *taptab = reinterpret_cast<int2 *>(biasl + 32 * MI + 4 * 32 * MI);     // [8 * Gp]
    float *stage = biasl + 32 * MI + 4 * 32 * MI + 16 * (G8 + kPwRing) + wave * (32 * kPwStageStride);   // a.wide_store

    // tiles gw, gw + NW, ... belong to this wave
    const int NW = gridDim.x * kPwWaves;
    const int gw = blockIdx.x * kPwWaves + wave;
    const int mytiles = gw < a.ntiles ? (a.ntiles - gw + NW - 1) / NW : 0;
    const int hwb = a.HW * 4;                    // bytes per channel plane

    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, a.in_bytes, 0x00020000);
    const int dlim = a.D - lhi;    // this lane's channel 8g + 2e + lhi exists iff 8g + 2e < dlim

    // byte offset of (pixel of this lane, channel lhi) of a tile; lanes past the last
    // pixel and tiles past the last one get an offset outside the buffer (loads give 0)
    // (straight-line arithmetic; an invalid lane only gets the top offset bit set)
    auto tile_voff = [&](int tile) -> uint32_t {
        const uint32_t m = (uint32_t)(tile * 32 + l32);
        const uint32_t bad = (tile < a.ntiles && m < (uint32_t)a.M) ? 0u : 0x80000000u;
        const uint32_t n = fast_div(m, a.div_HW);
        const uint32_t p = m - n * (uint32_t)a.HW;
        return ((((n * (uint32_t)a.D + (uint32_t)lhi) * (uint32_t)a.HW + p) * 4u) & 0x7fffffffu) | bad;
    };

    // Ring of loaded 8-channel groups: group g of a tile always lives in slot g % ring
    // size, so that the slot of every MFMA operand is fixed at compile time.  A tile is
    // treated as Gp = G8 rounded up to the ring size groups; the padding groups are
    // fetched with offsets outside the buffer (no memory traffic) and their MFMAs are
    // skipped.  That keeps the number of loads between a slot's fill and its use the same
    // on every path, so the wait before the use can leave the younger loads in flight.
    // When group g is consumed its slot is refilled with group g + ring size of the same
    // tile, or, past Gp, with group g % ring size of the wave's next tile.
    // Only the last group of a tile can hold channels past D; its per-lane invalid bits
    // are kept in four registers and switched on by a wave-uniform mask, which costs one
    // instruction per load.
    float b[RING][4];
    uint32_t lastbad[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) lastbad[e] = ((G8 - 1) * 8 + 2 * e < dlim) ? 0u : 0x80000000u;
    auto issue = [&](int u, uint32_t voff, int grp) {
        const uint32_t is_last = grp == G8 - 1 ? 0xffffffffu : 0u;     // wave-uniform
        const uint32_t gbad = grp < G8 ? 0u : 0x80000000u;             // padding group: nothing to fetch
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int d0 = grp * 8 + 2 * e;
            const uint32_t off = (lastbad[e] & is_last) | voff | gbad;
            b[u][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, d0 * hwb, 0));
        }
    };
    // TAPS: what a tile needs for its loads: the byte offset of the lane's window origin
    // (negative when the window starts in the padding: such an offset has bit 31 set and is
    // out of range by itself; a lane without a pixel gets bit 31 as well) and the complement
    // of the lane's set of valid taps, bit r for window row r and bit 16 + t for window column
    // t.  Bit 15 is never a valid row: table entries past the depth (the rest of the last
    // group, the padding groups of the ring) carry it and so never fetch.
    struct TapTile {
        int base;
        uint32_t nvalid;
    };
    auto range_mask = [](int lo, int hi) -> uint32_t {        // bits lo .. hi-1, lo >= 0, hi <= 15
        return hi > lo ? ((1u << hi) - 1u) & ~((1u << lo) - 1u) : 0u;
    };
    auto tap_tile = [&](int tile) -> TapTile {
        TapTile tt;
        const uint32_t m = (uint32_t)(tile * 32 + l32);
        const bool mv = tile < a.ntiles && m < (uint32_t)a.M;
        const uint32_t mm = mv ? m : 0u;
        const int n = (int)fast_div(mm, a.div_HW), pq = (int)mm - n * a.HW;
        const int p = (int)fast_div((uint32_t)pq, a.div_tQ), q = pq - p * a.tQ;
        const int ih0 = p * a.tsh - a.tph, iw0 = q * a.tsw - a.tpw;
        tt.base = (((n * a.tC * a.tH + ih0) * a.tW + iw0) * 4) | (mv ? 0 : (int)0x80000000);
        const uint32_t rows = range_mask(max(0, -ih0), min(a.tR, a.tH - ih0));
        const uint32_t cols = range_mask(max(0, -iw0), min(a.tS, a.tW - iw0));
        tt.nvalid = ~(rows | (cols << 16));
        return tt;
    };
    auto issue_taps = [&](int u, const TapTile &tt, int grp) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int2 tp = taptab[grp * 8 + 2 * e + lhi];
            // (straight-line: a select between the sum and a constant turns into a branch
            // around the LDS read of the offset)
            const uint32_t off = (uint32_t)(tt.base + tp.x) | (((uint32_t)tp.y & tt.nvalid) ? 0x80000000u : 0u);
            b[u][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0));
        }
    };
    uint32_t cur_voff = TAPS ? 0u : tile_voff(gw);
    // the first loads go out before the LDS fill (not TAPS: they need the tap table)
    // (in slot order, and kept in that order: the wait before a slot's first use counts
    // the loads issued after the slot's own)
    if (!TAPS) {
#pragma unroll
        for (int u = 0; u < RING; ++u) {
            issue(u, cur_voff, u);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- A and the bias to LDS ----
    const int a_floats = G8 * MI * kPwBlk;
    for (int i = tid * 4; i < a_floats; i += 4 * kPwThreads) *reinterpret_cast<floatx4 *>(&lds[i]) = floatx4{0.f, 0.f, 0.f, 0.f};
    auto row_group = [&](int r) -> int {
        return GROUPED ? (r >= a.r0[1]) + (r >= a.r0[2]) + (r >= a.r0[3]) : 0;
    };
    for (int r = tid; r < 32 * MI; r += kPwThreads) {
        float v = 0.f;
        if (r < a.Rout) {
            const int g = row_group(r);
            const float *bp = g == 0 ? a.bias[0] : g == 1 ? a.bias[1] : g == 2 ? a.bias[2] : a.bias[3];
            const int rb = g == 0 ? a.r0[0] : g == 1 ? a.r0[1] : g == 2 ? a.r0[2] : a.r0[3];
            if (bp) v = bp[r - rb];
            if (GROUPED) {
                float *o = g == 0 ? a.out[0] : g == 1 ? a.out[1] : g == 2 ? a.out[2] : a.out[3];
                const int re = g == 0 ? a.r0[1] : g == 1 ? a.r0[2] : g == 2 ? a.r0[3] : a.r0[4];
                RowDst rd;
                rd.base = o + (int64_t)(r - rb) * a.HW;
                rd.img_stride = (re - rb) * a.HW;
                rd.unused = 0;
                rowdst[r] = rd;
            }
        }
        biasl[r] = v;
    }
    __syncthreads();
    // walk A in memory order (coalesced), scatter into operand order; all of a thread's
    // loads of a pass are in flight together, since every workgroup waits for this
    // before its first MFMA
    {
        const int total = a.Rout * a.D;
        const bool depth_fast = a.depth_fast != 0;
        auto lds_index = [&](int r, int d) -> int {
            return ((d >> 3) * MI + (r >> 5)) * kPwBlk + (((d & 1) << 5) + (r & 31)) * 4 + ((d & 7) >> 1);
        };
        // memory index -> x = row, y = depth (branch-free: the quotient and remainder by
        // the contiguous axis, swapped for the transposed operand)
        auto split_index = [&](int idx) -> int2 {
            if (TAPS && a.tap_bwd) {
                // w[k][c][r][t] walked in memory order: row c, depth (k, r, t)
                const int RS = a.tR * a.tS;
                const int kc = (int)fast_div((uint32_t)idx, a.div_tRS), rs = idx - kc * RS;
                const int k = (int)fast_div((uint32_t)kc, a.div_rows), c = kc - k * a.Rout;
                return make_int2(c, k * RS + rs);
            }
            const int q = (int)fast_div((uint32_t)idx, a.div_fast);
            const int rem = idx - q * (depth_fast ? a.D : a.Rout);
            return depth_fast ? make_int2(q, rem) : make_int2(rem, q);
        };
        auto source = [&](int r, int d) -> const float * {
            const int g = row_group(r);
            const float *wp = g == 0 ? a.w[0] : g == 1 ? a.w[1] : g == 2 ? a.w[2] : a.w[3];
            const int rb = g == 0 ? a.r0[0] : g == 1 ? a.r0[1] : g == 2 ? a.r0[2] : a.r0[3];
            return wp + (r - rb) * a.w_row_stride + d * a.w_depth_stride;
        };
        if (a.fill_vec) {
            // four consecutive elements of the fast axis per load (aligned, same group)
            constexpr int FB = 8;
            const int total4 = total >> 2;
            for (int base = tid; base < total4; base += kPwThreads * FB) {
                floatx4 v[FB];
                int rr[FB], dd[FB];
#pragma unroll
                for (int j = 0; j < FB; ++j) {
                    const int i4 = base + j * kPwThreads;
                    rr[j] = -1;
                    dd[j] = 0;
                    v[j] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (i4 < total4) {
                        const int2 rd = split_index(i4 * 4);
                        v[j] = *reinterpret_cast<const floatx4 *>(source(rd.x, rd.y));
                        rr[j] = rd.x;
                        dd[j] = rd.y;
                    }
                }
                // the four elements share a block: depths d..d+3 (d % 4 == 0) are the two
                // half-waves of two consecutive vector elements, rows r..r+3 four lanes
#pragma unroll
                for (int j = 0; j < FB; ++j)
                    if (rr[j] >= 0) {
                        float *dst = &lds[lds_index(rr[j], dd[j])];
                        if (depth_fast) {
                            dst[0] = v[j][0]; dst[128] = v[j][1]; dst[1] = v[j][2]; dst[129] = v[j][3];
                        } else {
                            dst[0] = v[j][0]; dst[4] = v[j][1]; dst[8] = v[j][2]; dst[12] = v[j][3];
                        }
                    }
            }
        } else {
            constexpr int FB = 16;
            for (int base = tid; base < total; base += kPwThreads * FB) {
                float v[FB];
                int dst[FB];
#pragma unroll
                for (int j = 0; j < FB; ++j) {
                    const int idx = base + j * kPwThreads;
                    dst[j] = -1;
                    v[j] = 0.f;
                    if (idx < total) {
                        const int2 rd = split_index(idx);
                        v[j] = (TAPS && a.tap_bwd) ? a.w[0][idx] : *source(rd.x, rd.y);
                        dst[j] = lds_index(rd.x, rd.y);
                    }
                }
#pragma unroll
                for (int j = 0; j < FB; ++j)
                    if (dst[j] >= 0) lds[dst[j]] = v[j];
            }
        }
    }
    if (TAPS) {
        for (int d = tid; d < 8 * Gp; d += kPwThreads) {
            int2 e = make_int2(0, 1 << 15);                    // past D: never fetched
            if (d < a.D) {
                const int RS = a.tR * a.tS;
                const int c = d / RS, rs = d - c * RS;
                int r = rs / a.tS, t = rs - r * a.tS;
                if (a.tap_bwd) {                               // backward-data: the filter is flipped
                    r = a.tR - 1 - r;
                    t = a.tS - 1 - t;
                }
                e = make_int2(((c * a.tH + r) * a.tW + t) * 4, (1 << r) | (1 << (16 + t)));
            }
            taptab[d] = e;
        }
    }
    __syncthreads();
    TapTile cur_tt = {}, next_tt = {};
    if (TAPS) {
        cur_tt = tap_tile(gw);
#pragma unroll
        for (int u = 0; u < RING; ++u) {
            issue_taps(u, cur_tt, u);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // the accumulators start from the bias of their rows (0 without one)
    floatx16 acc[MI];
    auto init_acc = [&]() {
        asm volatile("" ::: "memory");
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 bv = *reinterpret_cast<const floatx4 *>(&biasl[32 * mi + 8 * q + 4 * lhi]);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[mi][4 * q + i] = bv[i];
            }
    };
    init_acc();

    const __amdgpu_buffer_rsrc_t orsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.out[0], 0, a.out_bytes, 0x00020000);
    auto store_tile = [&](int tile) {
        // the per-row values in LDS are re-read for every tile: kept in registers across
        // the main loop (they never change) they would crowd out the operand ring
        asm volatile("" ::: "memory");
        const int m = tile * 32 + l32;
        const bool mv = m < a.M;
        const int mm = mv ? m : 0;
        const int n = (int)fast_div((uint32_t)mm, a.div_HW);
        const int p = mm - n * a.HW;
        if (!GROUPED && a.wide_store) {
            // lane -> (row srow of an 8-row slab, pixels 4*sq .. 4*sq+3)
            const int sq = lane & 7, srow = lane >> 3;
            const int m4 = tile * 32 + 4 * sq;
            const bool mv4 = m4 < a.M;
            const int mm4 = mv4 ? m4 : 0;
            const int n4 = (int)fast_div((uint32_t)mm4, a.div_HW);
            const int p4 = mm4 - n4 * a.HW;
            const uint32_t voff = mv4 ? (uint32_t)((n4 * a.Rout + srow) * a.HW + p4) * 4u : 0x80000000u;
            float *wr = stage + (4 * lhi) * kPwStageStride + l32;
            const float *rd = stage + srow * kPwStageStride + 4 * sq;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int v = 0; v < 16; ++v) wr[(8 * (v >> 2) + (v & 3)) * kPwStageStride] = acc[mi][v];
                const bool full = 32 * mi + 32 <= a.Rout;      // wave-uniform
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    floatx4 val = *reinterpret_cast<const floatx4 *>(&rd[8 * it * kPwStageStride]);
                    if (a.relu) { val[0] = fmaxf(val[0], 0.f); val[1] = fmaxf(val[1], 0.f); val[2] = fmaxf(val[2], 0.f); val[3] = fmaxf(val[3], 0.f); }
                    // The row offset is added into the lane offset, not passed as the scalar
                    // offset: with a scalar-register offset the compiler assumes that the
                    // data registers of a 16-byte store may be overwritten by the very next
                    // vector instruction, and on this chip that store then wrote the new
                    // value of its first register from some lanes (seen as sporadic wrong
                    // first pixels of a quad).  In this form the compiler keeps the distance.
                    const uint32_t off = (full || 32 * mi + 8 * it + srow < a.Rout)
                                             ? voff + (uint32_t)((32 * mi + 8 * it) * hwb) : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) uint32_t, val),
                                                           orsrc, off, 0, 0);
                }
            }
        } else if (!GROUPED) {
            // rows 4*lhi + {0,1,2,3, 8,9,10,11, ...}: the row offset is wave-uniform (scalar
            // offset operand); a lane without a pixel stays outside the buffer
            const uint32_t off = mv ? (uint32_t)((n * a.Rout + 4 * lhi) * a.HW + p) * 4u : 0x80000000u;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const bool full = 32 * mi + 32 <= a.Rout;      // wave-uniform: every row of the tile exists
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r0 = 32 * mi + 8 * (v >> 2) + (v & 3);
                    float val = acc[mi][v];            // (a bit cast of the vector element itself takes element 0)
                    if (a.relu) val = fmaxf(val, 0.f);
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), orsrc,
                                                          (full || r0 + 4 * lhi < a.Rout) ? off : 0x80000000u,
                                                          r0 * hwb, 0);
                }
            }
        } else {
            // per-row records at compile-time offsets from a lane-dependent LDS address
            // (rows 4*lhi + ...); a global-memory store: a generic one
            // would make the waits for the loads in flight wait for everything
            typedef __attribute__((address_space(1))) float gfloat;
            const RowDst *rd0 = rowdst + 4 * lhi;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                if (32 * mi + 32 <= a.Rout) {      // wave-uniform: every row of the tile exists
                    if (mv) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int rr = 32 * mi + 8 * (v >> 2) + (v & 3);
                            const RowDst rd = rd0[rr];
                            ((gfloat *)rd.base)[n * rd.img_stride + p] = acc[mi][v];
                        }
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int rr = 32 * mi + 8 * (v >> 2) + (v & 3);
                        if (mv && rr + 4 * lhi < a.Rout) {
                            const RowDst rd = rd0[rr];
                            ((gfloat *)rd.base)[n * rd.img_stride + p] = acc[mi][v];
                        }
                    }
                }
            }
        }
    };

    // A operands: two register sets used alternately (unit u reads set u % 2 and fetches
    // the next group into the other one).  The first group of a tile is read from set 0:
    // after a tile with an odd number of groups it is moved there from set 1.
    floatx4 av[2][MI];
    if (mytiles > 0) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) av[0][mi] = *reinterpret_cast<const floatx4 *>(&lds[mi * kPwBlk + lane * 4]);
    }
    for (int t = 0, tile = gw; t < mytiles; ++t, tile += NW) {
        const uint32_t next_voff = TAPS ? 0u : tile_voff(tile + NW);
        if (TAPS) next_tt = tap_tile(tile + NW);
        for (int g0 = 0; g0 < Gp; g0 += RING) {
#pragma unroll
            for (int u = 0; u < RING; ++u) {
                const int g = g0 + u;
                if (g < G8) {
                    const int ng = (g + 1 == G8) ? 0 : g + 1;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        av[(u & 1) ^ 1][mi] =
                            *reinterpret_cast<const floatx4 *>(&lds[(ng * MI + mi) * kPwBlk + lane * 4]);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
                            acc[mi] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u & 1][mi][e], b[u][e], acc[mi], 0, 0, 0);
                }
                // the refill is issued on every path, also after a padding group
                const bool same = g + RING < Gp;
                if (TAPS) {
                    TapTile tt;
                    tt.base = same ? cur_tt.base : next_tt.base;
                    tt.nvalid = same ? cur_tt.nvalid : next_tt.nvalid;
                    issue_taps(u, tt, same ? g + RING : u);
                } else {
                    issue(u, same ? cur_voff : next_voff, same ? g + RING : u);
                }
            }
        }
        if (G8 & 1) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) av[0][mi] = av[1][mi];
        }
        store_tile(tile);
        cur_voff = next_voff;
        if (TAPS) cur_tt = next_tt;
        init_acc();
    }
}

template <int MI, bool GROUPED, bool TAPS = false, int RING = kPwRing>
static hipError_t launch_pw_stream_t(const PwArgs &a, size_t lds_bytes, int grid, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t cfg = hipSuccess;
    std::call_once(once, [] {
        cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(pw_stream_kernel<MI, GROUPED, TAPS, RING>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPwLdsMax);
    });
    if (cfg != hipSuccess) return cfg;
    const ProfScope ps(TAPS ? KID_TAP_STREAM : KID_PW_STREAM, 2.0 * a.M * (double)a.D * a.Rout,
                       (double)a.in_bytes + 4.0 * a.M * (double)a.Rout + 4.0 * a.D * (double)a.Rout, s);
    hipLaunchKernelGGL((pw_stream_kernel<MI, GROUPED, TAPS, RING>), dim3((unsigned)grid), dim3(kPwThreads), lds_bytes, s, a);
    return hipGetLastError();
}

// taps form: forward pass of a layer with at most 128 filters whose filter bank fits in LDS
// 16-byte stores need groups of four pixels that stay inside one image and are aligned,
// and room for the staging area beside A
static bool pw_wide_store(const PwArgs &a, size_t lds_bytes)
{
    return a.ngroup == 1 && a.HW % 4 == 0 && ((uintptr_t)a.out[0] & 15) == 0 && lds_bytes + kPwStageBytes <= kPwLdsMax;
}

hipError_t launch_tap_stream(const PwArgs &a0, hipStream_t s)
{
    PwArgs a = a0;
    size_t lds_bytes = pw_stream_lds_bytes(a.Rout, a.D);
    if (lds_bytes == 0 || a.Rout > 128 || a.ngroup != 1 || a.D != a.tC * a.tR * a.tS) return hipErrorInvalidValue;
    if (a.tap_bwd && a.fill_vec) return hipErrorInvalidValue;
    a.wide_store = pw_wide_store(a, lds_bytes);
    if (a.wide_store) lds_bytes += kPwStageBytes;
    int grid = (a.ntiles + kPwWaves - 1) / kPwWaves;
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    // at most 32 taps (3x3 over 3 channels): a ring of four groups holds a whole tile
    const bool small = a.D <= 32;
    switch (pw_row_tiles(a.Rout)) {
#define TAP_CASE(M)                                                                          \
    case M:                                                                                  \
        return small ? launch_pw_stream_t<M, false, true, 4>(a, lds_bytes, grid, s)          \
                     : launch_pw_stream_t<M, false, true>(a, lds_bytes, grid, s);
        TAP_CASE(1)
        TAP_CASE(2)
        TAP_CASE(3)
        TAP_CASE(4)
#undef TAP_CASE
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_pw_stream(const PwArgs &a0, hipStream_t s)
{
    PwArgs a = a0;
    size_t lds_bytes = pw_stream_lds_bytes(a.Rout, a.D);
    if (lds_bytes == 0) return hipErrorInvalidValue;
    a.wide_store = pw_wide_store(a, lds_bytes);
    if (a.wide_store) lds_bytes += kPwStageBytes;
    // one workgroup of eight waves per compute unit; a wave loops over its tiles
    int grid = (a.ntiles + kPwWaves - 1) / kPwWaves;
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    const bool grouped = a.ngroup > 1;
    switch (pw_row_tiles(a.Rout)) {
#define PW_CASE(M)                                                                           \
    case M:                                                                                  \
        return grouped ? launch_pw_stream_t<M, true>(a, lds_bytes, grid, s)                 \
                       : launch_pw_stream_t<M, false>(a, lds_bytes, grid, s);
        PW_CASE(1)
        PW_CASE(2)
        PW_CASE(3)
        PW_CASE(4)
        PW_CASE(6)
        PW_CASE(8)
#undef PW_CASE
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------- backward-weight ---
// The pixels are the reduction axis and both operands have them contiguous.  With
// v_mfma_f32_16x16x4_f32 (lane l supplies A[i = l%16][kk = l/16] and B[kk = l/16][j =
// l%16]; accumulator register v of lane l is row 4*(l/16) + v, column l%16) a lane
// fetches 16 bytes = 4 consecutive pixels of "its" row (filter 16*ai + l%16 of dy,
// channel 16*bj + l%16 of x) and the four lane groups l/16 take four consecutive groups
// of 4 pixels: one load per 16-row block covers 16 pixels, 64 contiguous bytes per row,
// and feeds 4 MFMAs per block pair (MFMA e contracts element e of the vectors: depth
// index kk stands for pixel 16*step + 4*kk + e, the same assignment on both operands).
// The number of cache lines a load touches, not its bytes, is what the vector memory
// pipe charges for here, so a wave computes a block of AT x BT accumulator tiles (AT
// covers all filters; the channels are spread over NJ waves), which keeps the loads per
// MFMA and the re-reads of dy by the other waves low.  x is read once from HBM, dy once
// from HBM and NJ - 1 times from the caches.
//
// Workgroup = NJ column groups x PH pixel phases, one wave each (phase ph takes the
// steps ph, ph + PH, ... of the workgroup's range); the phases' results are added
// through LDS at the end, in phase order.  The pixel axis is cut into `splits` ranges;
// each workgroup writes its partial K x C product (and column group 0 its partial bias
// gradient), added up by the split-reduce kernel.
//
// TAPS: the same kernel for a small stride-1 filter over very few channels (first layers:
// C*R*S <= 32).  The B rows are then the taps (c, r, s) of the lowered matrix instead of
// channels: lane l%16 owns tap t and fetches x[n][c_t][p + r_t - pad_h][q + s_t - pad_w + e],
// e = 0..3, with four dword loads (the shifted vector is not 16-byte aligned and its ends
// may fall into the padding: each element carries its own validity); dy, the accumulators,
// the phases and the output part[s][k][t] (= KCRS order) are unchanged.  Needs Q % 4 == 0.
template <int AT, int BT, bool TAPS>
__global__ __launch_bounds__(512) void pw_wgrad_kernel(PwWgradArgs a)
{
    constexpr int R = AT + BT <= 4 ? 4 : (AT + BT <= 6 ? 3 : 2);     // 16-pixel steps in flight
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int split = blockIdx.x;
    const int NJ = a.tiles_c, PH = a.phases;
    const int nj = wave % NJ, ph = wave / NJ;
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc((void *)a.dy, 0, a.dy_bytes, 0x00020000);

    // per-lane row offsets (elements) and invalid bits; an invalid access only gets the
    // top offset bit set, which puts it outside the buffer (valid offsets are below 2^31)
    uint32_t koff[AT], kbad[AT], coff[BT], cbad[BT];
#pragma unroll
    for (int ai = 0; ai < AT; ++ai) {
        const int k = 16 * ai + l16;
        kbad[ai] = k < a.K ? 0u : 0x80000000u;
        koff[ai] = (uint32_t)(k * a.HW);
    }
    int tdr[BT], tds[BT];             // TAPS: row / column displacement of this lane's tap
#pragma unroll
    for (int bj = 0; bj < BT; ++bj) {
        const int c = (nj * BT + bj) * 16 + l16;
        cbad[bj] = c < a.C ? 0u : 0x80000000u;
        if (TAPS) {
            const int cc = c < a.C ? c : 0;
            const int ch = (int)fast_div((uint32_t)cc, a.div_RS), rs = cc - ch * a.tR * a.tS;
            const int r = (int)fast_div((uint32_t)rs, a.div_S), t = rs - r * a.tS;
            tdr[bj] = r - a.tph;
            tds[bj] = t - a.tpw;
            coff[bj] = (uint32_t)(ch * a.xH * a.xW);
        } else {
            tdr[bj] = 0;
            tds[bj] = 0;
            coff[bj] = (uint32_t)(c * a.HW);
        }
    }
    const int xCHW = a.xC * a.xH * a.xW;      // TAPS: image stride of x
    const int QW = a.HW >> 2;
    const int KHW = a.K * a.HW, CHW = a.C * a.HW;
    const int total_steps = (a.quads + 3) >> 2;
    const int step0 = split * a.steps_per_split;
    int range = total_steps - step0;
    if (range > a.steps_per_split) range = a.steps_per_split;
    if (range < 0) range = 0;
    const int step_end = step0 + range;
    const int nsteps = range > ph ? (range - ph + PH - 1) / PH : 0;     // steps of this phase

    // Prefetch cursor: step pstep, and for this lane's 4-pixel group of that step its image
    // pn and pixel pp, kept up to date by additions (a step of this phase moves 16 * PH
    // pixels on: at most one image boundary, since H*W >= 16 * PH).
    floatx4 ar[R][AT], br[R][BT];
    int pstep = step0 + ph;
    int pn, pp;
    {
        const int qd = pstep * 4 + lq;
        pn = (int)fast_div((uint32_t)qd, a.div_QW);
        pp = (qd - pn * QW) * 4;
    }
    uint32_t dyb = (uint32_t)(pn * KHW + pp), xb = (uint32_t)(pn * CHW + pp);
    const int adv = 16 * PH;
    auto issue = [&](int u) {
        const uint32_t sbad = pstep < step_end ? 0u : 0x80000000u;          // wave-uniform
        const uint32_t qbad = (pn < a.N ? 0u : 0x80000000u) | sbad;
#pragma unroll
        for (int ai = 0; ai < AT; ++ai)
            ar[u][ai] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                        rs_dy, (((dyb + koff[ai]) * 4u) & 0x7fffffffu) | qbad | kbad[ai], 0, 0));
        if (TAPS) {
            const int p = (int)fast_div((uint32_t)pp, a.div_Q), q0 = pp - p * a.Qd;
            const int img = pn * xCHW;
#pragma unroll
            for (int bj = 0; bj < BT; ++bj) {
                const int row = p + tdr[bj], col0 = q0 + tds[bj];
                const uint32_t rbad = ((unsigned)row < (unsigned)a.xH ? 0u : 0x80000000u) | qbad | cbad[bj];
                const int base = img + (int)coff[bj] + row * a.xW + col0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t ebad = (unsigned)(col0 + e) < (unsigned)a.xW ? 0u : 0x80000000u;
                    br[u][bj][e] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(
                                   rs_x, (((uint32_t)(base + e) * 4u) & 0x7fffffffu) | rbad | ebad, 0, 0));
                }
            }
        } else {
#pragma unroll
            for (int bj = 0; bj < BT; ++bj)
                br[u][bj] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                            rs_x, (((xb + coff[bj]) * 4u) & 0x7fffffffu) | qbad | cbad[bj], 0, 0));
        }
        pstep += PH;
        pp += adv;
        const bool wrap = pp >= a.HW;
        pp -= wrap ? a.HW : 0;
        pn += wrap ? 1 : 0;
        dyb += (uint32_t)(wrap ? adv + KHW - a.HW : adv);
        xb += (uint32_t)(wrap ? adv + CHW - a.HW : adv);
    };
    // in slot order, and kept in that order: the wait before a slot's first use counts
    // the loads issued after the slot's own
#pragma unroll
    for (int u = 0; u < R; ++u) {
        issue(u);
        __builtin_amdgcn_sched_barrier(0);
    }

    floatx4 acc[AT][BT];
    float bsum[AT];
#pragma unroll
    for (int ai = 0; ai < AT; ++ai) {
        bsum[ai] = 0.f;
#pragma unroll
        for (int bj = 0; bj < BT; ++bj) acc[ai][bj] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const bool want_bias = a.bias_part != nullptr && nj == 0;

    for (int it = 0; it < nsteps; it += R) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            if (it + u < nsteps) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int ai = 0; ai < AT; ++ai)
#pragma unroll
                        for (int bj = 0; bj < BT; ++bj)
                            acc[ai][bj] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[u][ai][e], br[u][bj][e], acc[ai][bj], 0, 0, 0);
                if (want_bias) {
#pragma unroll
                    for (int ai = 0; ai < AT; ++ai)
                        bsum[ai] += (ar[u][ai][0] + ar[u][ai][1]) + (ar[u][ai][2] + ar[u][ai][3]);
                }
            }
            // refill on every path (past the range: offsets outside the buffers), so that
            // the count of loads between a slot's fill and its use does not depend on the path
            issue(u);
        }
    }

    // ---- phases 1.. hand their sums to phase 0 through LDS ----
    // layout: [ph - 1][nj][(ai * BT + bj) * 4 + v][lane], then the bias sums [ph - 1][ai][lane]
    constexpr int ACC = AT * BT * 4;
    if (PH > 1) {
        float *bl = lds + (PH - 1) * NJ * ACC * 64;
        if (ph > 0) {
            float *dst = lds + ((ph - 1) * NJ + nj) * ACC * 64;
#pragma unroll
            for (int ai = 0; ai < AT; ++ai)
#pragma unroll
                for (int bj = 0; bj < BT; ++bj)
#pragma unroll
                    for (int v = 0; v < 4; ++v) dst[((ai * BT + bj) * 4 + v) * 64 + lane] = acc[ai][bj][v];
            if (nj == 0) {
#pragma unroll
                for (int ai = 0; ai < AT; ++ai) bl[((ph - 1) * AT + ai) * 64 + lane] = bsum[ai];
            }
        }
        __syncthreads();
        if (ph > 0) return;
        for (int q = 1; q < PH; ++q) {
            const float *src = lds + ((q - 1) * NJ + nj) * ACC * 64;
#pragma unroll
            for (int ai = 0; ai < AT; ++ai)
#pragma unroll
                for (int bj = 0; bj < BT; ++bj)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[ai][bj][v] += src[((ai * BT + bj) * 4 + v) * 64 + lane];
            if (nj == 0) {
#pragma unroll
                for (int ai = 0; ai < AT; ++ai) bsum[ai] += bl[((q - 1) * AT + ai) * 64 + lane];
            }
        }
    }

    float *out = a.part + (int64_t)split * a.K * a.C;
#pragma unroll
    for (int bj = 0; bj < BT; ++bj) {
        const int c = (nj * BT + bj) * 16 + l16;
        if (c >= a.C) continue;
#pragma unroll
        for (int ai = 0; ai < AT; ++ai)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = 16 * ai + 4 * lq + v;
                if (k < a.K) out[k * a.C + c] = acc[ai][bj][v];
            }
    }
    if (want_bias) {
#pragma unroll
        for (int ai = 0; ai < AT; ++ai) {
            float v = bsum[ai];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            const int k = 16 * ai + l16;
            if (lq == 0 && k < a.K) a.bias_part[split * a.K + k] = v;
        }
    }
}

constexpr size_t kPwWgradLdsMax = 128 * 1024;

static int pw_wgrad_at(int K)
{
    const int t = (K + 15) / 16;
    return t <= 4 ? t : (t <= 6 ? 6 : 8);
}

// Shape of the workgroup for C channels and K filters: column groups NJ (1, 2, 4 or 8) of BT
// 16-channel tiles each, and the pixel phases: as many (a power of two) as keep the
// workgroup within eight waves, a step of all phases within one image (16 * PH <= HW) and
// the phase sums within the LDS limit.
void pw_wgrad_shape(int C, int K, int HW, int *NJ, int *BT, int *PH)
{
    const int cb = (C + 15) / 16;
    const int at = pw_wgrad_at(K);
    int nj = cb <= 4 ? 1 : (cb <= 8 ? 2 : 4);
    int bt = (cb + nj - 1) / nj;
    if (at == 8 && bt == 4) {        // 8 x 4 accumulator tiles do not fit the registers of a wave
        nj *= 2;
        bt = 2;
    }
    if (bt < 2) bt = 2;
    int ph = 8 / nj;
    while (ph > 1 && (16 * ph > HW ||
                      (size_t)(ph - 1) * (nj * at * bt * 4 + at) * 64 * sizeof(float) > kPwWgradLdsMax))
        ph >>= 1;
    *NJ = nj;
    *BT = bt;
    *PH = ph;
}

template <int AT, int BT, bool TAPS = false>
static hipError_t launch_pw_wgrad_t(const PwWgradArgs &a, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t cfg = hipSuccess;
    std::call_once(once, [] {
        cfg = hipFuncSetAttribute(reinterpret_cast<const void *>(pw_wgrad_kernel<AT, BT, TAPS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPwWgradLdsMax);
    });
    if (cfg != hipSuccess) return cfg;
    const ProfScope ps(TAPS ? KID_TAP_WGRAD : KID_PW_WGRAD, 2.0 * a.N * (double)a.HW * a.C * a.K,
                       (double)a.x_bytes + (double)a.dy_bytes + 4.0 * a.K * (double)a.C, s);
    hipLaunchKernelGGL((pw_wgrad_kernel<AT, BT, TAPS>), grid, block, lds_bytes, s, a);
    return hipGetLastError();
}

template <int AT>
static hipError_t launch_pw_wgrad_bt(const PwWgradArgs &a, int BT, dim3 grid, dim3 block, size_t lds_bytes,
                                     hipStream_t s)
{
    switch (BT) {
    case 2: return launch_pw_wgrad_t<AT, 2>(a, grid, block, lds_bytes, s);
    case 3: return launch_pw_wgrad_t<AT, 3>(a, grid, block, lds_bytes, s);
    case 4: return launch_pw_wgrad_t<AT, 4>(a, grid, block, lds_bytes, s);
    default: return hipErrorInvalidValue;
    }
}

// TAPS form: a.C = number of taps (<= 32: one column group of two 16-tap tiles), a.HW = P*Q
hipError_t launch_tap_wgrad(const PwWgradArgs &a, hipStream_t s)
{
    if (a.K < 1 || a.K > 128 || a.C < 1 || a.C > 32 || a.splits < 1 || a.Qd % 4 != 0 || a.HW != a.tP * a.Qd)
        return hipErrorInvalidValue;
    int NJ, BT, PH;
    pw_wgrad_shape(a.C, a.K, a.HW, &NJ, &BT, &PH);
    if (NJ != 1 || BT != 2 || a.tiles_c != NJ || a.phases != PH || a.HW < 16 * PH) return hipErrorInvalidValue;
    const int AT = pw_wgrad_at(a.K);
    const dim3 grid((unsigned)a.splits), block((unsigned)(64 * NJ * PH));
    const size_t lds_bytes = (size_t)(PH - 1) * (NJ * AT * BT * 4 + AT) * 64 * sizeof(float);
    switch (AT) {
    case 1: return launch_pw_wgrad_t<1, 2, true>(a, grid, block, lds_bytes, s);
    case 2: return launch_pw_wgrad_t<2, 2, true>(a, grid, block, lds_bytes, s);
    case 3: return launch_pw_wgrad_t<3, 2, true>(a, grid, block, lds_bytes, s);
    case 4: return launch_pw_wgrad_t<4, 2, true>(a, grid, block, lds_bytes, s);
    case 6: return launch_pw_wgrad_t<6, 2, true>(a, grid, block, lds_bytes, s);
    default: return launch_pw_wgrad_t<8, 2, true>(a, grid, block, lds_bytes, s);
    }
}

hipError_t launch_pw_wgrad(const PwWgradArgs &a, hipStream_t s)
{
    if (a.K < 1 || a.K > 128 || a.C < 1 || a.C > 256 || a.splits < 1 || a.HW % 4 != 0) return hipErrorInvalidValue;
    int NJ, BT, PH;
    pw_wgrad_shape(a.C, a.K, a.HW, &NJ, &BT, &PH);
    if (a.tiles_c != NJ || a.phases != PH || a.HW < 16 * PH) return hipErrorInvalidValue;
    const int AT = pw_wgrad_at(a.K);
    const dim3 grid((unsigned)a.splits), block((unsigned)(64 * NJ * PH));
    const size_t lds_bytes = (size_t)(PH - 1) * (NJ * AT * BT * 4 + AT) * 64 * sizeof(float);
    switch (AT) {
    case 1: return launch_pw_wgrad_bt<1>(a, BT, grid, block, lds_bytes, s);
    case 2: return launch_pw_wgrad_bt<2>(a, BT, grid, block, lds_bytes, s);
    case 3: return launch_pw_wgrad_bt<3>(a, BT, grid, block, lds_bytes, s);
    case 4: return launch_pw_wgrad_bt<4>(a, BT, grid, block, lds_bytes, s);
    case 6: return launch_pw_wgrad_bt<6>(a, BT, grid, block, lds_bytes, s);
    default:
        if (BT == 2) return launch_pw_wgrad_t<8, 2>(a, grid, block, lds_bytes, s);
        if (BT == 3) return launch_pw_wgrad_t<8, 3>(a, grid, block, lds_bytes, s);
        return hipErrorInvalidValue;
    }
}

}  // namespace mi355conv
