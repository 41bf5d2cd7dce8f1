// Implicit-GEMM convolution on fp32 MFMA for gfx950: forward and backward-data.
//
// Sec. 4.2 "implicitgemm" of the paper: lower the convolution onto a matrix
// product but form the lowered matrix lazily in on-chip memory.  Here the
// product is  out[Kout x pixels] = Wt^T[Kout x depth] * lowered[depth x pixels]:
//   * filters are the MFMA "A" rows, output pixels the "B" columns, so that in
//     the 32x32 accumulator layout the 32 lanes of a half-wave hold 32
//     consecutive output pixels of one filter: NCHW stores are 128-byte rows;
//   * the lowered tile (kDepthTile rows x BN pixels) is gathered straight from
//     the NCHW tensor into LDS, lanes running along the pixel axis (W is the
//     contiguous axis, so stride-1 gathers coalesce);
//   * the filter matrix is pre-transposed to [depth][Kpad] so its tiles are
//     plain 16-byte row reads;
//   * bias (and, on request, the ReLU that follows the layer) is applied in the epilogue
//     before the only store (the fused epilogue of Sec. 4.2 "Neon").
// 256 threads = 4 waves; LDS tiles are double buffered, one barrier per step.

#include "conv_internal.h"

#include <type_traits>

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ prep ---
// Writes the filter matrix Wt[row][col] (zero padded) and the gather table.
__global__ __launch_bounds__(256) void gemmconv_prep_kernel(PrepArgs a)
{
    const int64_t total = (int64_t)a.rows_total * a.Kpad;
    const int RS = a.R * a.S;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int row = (int)(i / a.Kpad);
        const int col = (int)(i - (int64_t)row * a.Kpad);
        int p = 0;
        while (p + 1 < a.nphases && row >= a.ph[p + 1].row0) ++p;
        const PrepPhase ph = a.ph[p];
        const int d = row - ph.row0;
        float v = 0.f;
        DepthEntry e;
        e.off = 0;
        e.drdt = kInvalidDr << 16;
        if (d < ph.rows) {
            if (a.mode == 0 || a.mode == 3) {
                // forward: row d = (c, r, t), column = filter k
                const int c = d / RS, rt = d - c * RS, r = rt / a.S, t = rt - r * a.S;
                e.off = c * a.gather_chan_stride + r * a.gather_W + t;
                e.drdt = (int32_t)(((uint32_t)r << 16) | ((uint32_t)t & 0xffffu));
                if (col < a.K) {
                    if (a.mode == 0) {
                        v = a.w[(int64_t)col * a.C * RS + d];
                    } else {
                        // stacked groups: column col is filter col - gk0[g] of group g
                        int g = 0;
                        while (g + 1 < kMaxGroups && col >= a.gk0[g + 1]) ++g;
                        const float *gw = g == 0 ? a.gw[0] : g == 1 ? a.gw[1] : g == 2 ? a.gw[2] : a.gw[3];
                        const int k0 = g == 0 ? a.gk0[0] : g == 1 ? a.gk0[1] : g == 2 ? a.gk0[2] : a.gk0[3];
                        v = gw[(int64_t)(col - k0) * a.C * RS + d];
                    }
                }
            } else if (a.mode == 2) {
                // backward-data, all phases at once: row d = (k, dr, dt) over the union of
                // the phases' tap displacements, column k' = (pa, pb, c): output pixel
                // (oh*sh + pa, ow*sw + pb) of channel c receives dy[oh + dr][ow + dt] through
                // the tap r = pa + pad_h - dr*sh, t = pb + pad_w - dt*sw (if that tap exists)
                const int ndd = a.nd_r * a.nd_t;
                const int k = d / ndd, rt = d - k * ndd, ir = rt / a.nd_t, it = rt - ir * a.nd_t;
                const int dr = a.dr_min + ir, dt = a.dt_min + it;
                e.off = k * a.gather_chan_stride + dr * a.gather_W + dt;
                e.drdt = (int32_t)(((uint32_t)dr << 16) | ((uint32_t)dt & 0xffffu));
                const int cols = a.stride_h * a.stride_w * a.C;
                if (col < cols) {
                    const int pab = col / a.C, c = col - pab * a.C;
                    const int pa = pab / a.stride_w, pb = pab - pa * a.stride_w;
                    const int r = pa + a.pad_h - dr * a.stride_h, t = pb + a.pad_w - dt * a.stride_w;
                    if (r >= 0 && r < a.R && t >= 0 && t < a.S)
                        v = a.w[(((int64_t)k * a.C + c) * a.R + r) * a.S + t];
                }
            } else {
                // backward-data: row d = (k, r', t') of this phase, column = channel c
                const int nrt = ph.nr * ph.nt;
                const int k = d / nrt, rt = d - k * nrt, ri = rt / ph.nt, ti = rt - ri * ph.nt;
                const int r = ph.r0 + ri * a.stride_h, t = ph.t0 + ti * a.stride_w;
                e.off = k * a.gather_chan_stride - ri * a.gather_W - ti;
                e.drdt = (int32_t)(((uint32_t)(-ri) << 16) | ((uint32_t)(-ti) & 0xffffu));
                if (col < a.C) v = a.w[(((int64_t)k * a.C + col) * a.R + r) * a.S + t];
            }
        }
        a.wt[i] = v;
        if (col == 0) a.tab[row] = e;
    }
}

hipError_t launch_gemmconv_prep(const PrepArgs &a, hipStream_t s)
{
    const int64_t total = (int64_t)a.rows_total * a.Kpad;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(gemmconv_prep_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ main ---
// XCD-aware block order: hardware deals consecutive workgroup ids round-robin to
// the 8 XCDs (each with its own L2).  Remap so every XCD works on one contiguous
// run of logical tiles; logical order has the filter tile fastest, so the blocks
// that gather the same pixels run next to each other on the same L2.
__device__ __forceinline__ int xcd_remap(int id, int nb)
{
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = id & 7, local = id >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}

// Workgroup barrier that orders LDS traffic only: global loads already in flight
// (the register prefetch of a later tile) are not waited for.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// PW ("pointwise"): 1x1 stride-1 unpadded layers whose H*W is a multiple of 4.
// The lowered tile is then a plain [channels x pixels] block of the tensor: it is
// fetched with 16-byte buffer loads (4 pixels of one channel per thread, fixed
// per-thread offsets, the depth step in the scalar offset) instead of per-element
// gathers, which is what lets these HBM-bound layers stream.
template <int BM, int BN, int WM, int WN, bool PW>
__global__ __launch_bounds__(256) void gemmconv_kernel(GemmConvArgs a)
{
    constexpr int BK = kDepthTile;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * WAVES_N == 4, "4 waves per workgroup");
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int TPP = 256 / BN;            // threads per pixel column: 1 or 2
    // elements fetched per thread and tile: gathered rows, or (PW) 4-pixel vectors
    constexpr int B_ROWS = PW ? BK * BN / 1024 : BK / TPP;
    constexpr int PW_VPR = BN / 4;           // PW: vectors per tile row
    constexpr int PW_RPP = 256 / PW_VPR;     // PW: rows per pass of the 256 threads
    constexpr int A_VECS = BK * BM / 4;      // float4 per filter tile
    constexpr int A_PER_THREAD = (A_VECS + 255) / 256;
    static_assert(BN >= 64 && 256 % BN == 0, "pixel tile");

    __shared__ float As[2][BK][BM];
    __shared__ float Bs[2][BK][BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const Phase ph = a.phase[blockIdx.y];

    const int logical = xcd_remap(blockIdx.x, gridDim.x);
    const int kt = logical % a.tiles_k;
    const int pt = logical / a.tiles_k;
    const int HWs = ph.Hs * ph.Ws;
    const int Mpix = a.N * HWs;
    if (pt * BN >= Mpix) return;             // phase with fewer pixel tiles

    // ---- gather set-up: this thread's pixel column ----
    const int pcol = tid % BN;
    const int prow0 = __builtin_amdgcn_readfirstlane(tid / BN);   // wave-uniform (BN >= 64)
    int gbase = 0, ih0 = -(1 << 24), iw0 = 0;
    {
        const int m = pt * BN + pcol;
        if (m < Mpix) {
            const int n = m / HWs, rem = m - n * HWs;
            const int oh = rem / ph.Ws, ow = rem - oh * ph.Ws;
            ih0 = oh * a.in_step_h + ph.in_base_h;
            iw0 = ow * a.in_step_w + ph.in_base_w;
            gbase = n * a.in_img_stride + ih0 * a.Win + iw0;
        }
    }
    const DepthEntry *tab = a.tab + ph.row0;
    const float *wt = a.wt + (int64_t)ph.row0 * a.Kpad + kt * BM;

    // PW set-up: this thread's 4 pixels and its rows of every depth tile
    const __amdgpu_buffer_rsrc_t pw_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.in, 0, PW ? a.in_bytes : 0, 0x00020000);
    const int pw_row0 = tid / PW_VPR, pw_col = (tid % PW_VPR) * 4;
    const int pw_chan_bytes = a.Hin * a.Win * 4;
    uint32_t pw_off[B_ROWS];
    if (PW) {
        const int m = pt * BN + pw_col;
        const int n = m / HWs, rem = m - n * HWs;          // the 4 pixels share an image (HW % 4 == 0)
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i)
            pw_off[i] = m < Mpix ? (uint32_t)(n * a.in_img_stride + rem) * 4u + (uint32_t)(pw_row0 + i * PW_RPP) * (uint32_t)pw_chan_bytes
                                 : 0x80000000u;
    }

    typename std::conditional<PW, floatx4, float>::type breg[B_ROWS];
    floatx4 areg[A_PER_THREAD];
    uint32_t bmask = 0;    // bit i: gathered element i is inside the image
    DepthEntry ent[B_ROWS];   // table rows of the tile being gathered (wave-uniform: SGPRs)

    // This thread gathers rows prow0*B_ROWS .. +B_ROWS-1 of a depth tile: one
    // contiguous run of table entries, fetched with wide scalar loads.
    int pw_depth0 = 0;       // PW: first channel of the tile being fetched
    auto table_fetch = [&](int tile) {
        if constexpr (PW) {
            pw_depth0 = tile * BK;
        } else {
#pragma unroll
            for (int i = 0; i < B_ROWS; ++i) ent[i] = tab[tile * BK + prow0 * B_ROWS + i];
        }
    };
    auto gather_issue = [&](int i) {
        if constexpr (PW) {
            // channels past the real depth (padding rows of the last tile) read as 0
            const uint32_t off = (pw_depth0 + pw_row0 + i * PW_RPP < a.pw_depth) ? pw_off[i] : 0x80000000u;
            breg[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                      pw_rsrc, off, pw_depth0 * pw_chan_bytes, 0));
            return;
        } else {
        const DepthEntry e = ent[i];
        const int dr = e.drdt >> 16;
        const int dt = (int)(short)(e.drdt & 0xffff);
        const bool ok = ((unsigned)(ih0 + dr) < (unsigned)a.Hin) &&
                        ((unsigned)(iw0 + dt) < (unsigned)a.Win);
        const int idx = ok ? gbase + e.off : 0;
        breg[i] = a.in[idx];
        bmask = (bmask & ~(1u << i)) | (ok ? (1u << i) : 0u);
        }
    };
    auto filter_issue = [&](int tile, int i) {
        const int vi = tid + i * 256;
        if (A_VECS % 256 == 0 || vi < A_VECS) {
            const int row = vi / (BM / 4), c4 = vi - row * (BM / 4);
            areg[i] = *reinterpret_cast<const floatx4 *>(wt + (int64_t)(tile * BK + row) * a.Kpad + c4 * 4);
        }
    };
    auto store_b = [&](int buf, int i) {
        if constexpr (PW) {
            *reinterpret_cast<floatx4 *>(&Bs[buf][pw_row0 + i * PW_RPP][pw_col]) = breg[i];
        } else {
            Bs[buf][prow0 * B_ROWS + i][pcol] = ((bmask >> i) & 1u) ? breg[i] : 0.f;
        }
    };
    auto store_a = [&](int buf, int i) {
        const int vi = tid + i * 256;
        if (A_VECS % 256 == 0 || vi < A_VECS) {
            const int row = vi / (BM / 4), c4 = vi - row * (BM / 4);
            *reinterpret_cast<floatx4 *>(&As[buf][row][c4 * 4]) = areg[i];
        }
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    const int wm0 = (wave / WAVES_N) * WM;
    const int wn0 = (wave % WAVES_N) * WN;
    const int l32 = lane & 31, lhi = lane >> 5;

    float av[2][MI], bv[2][NI];
    auto read_ops = [&](int buf, int kk, int slot) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) av[slot][mi] = As[buf][kk + lhi][wm0 + mi * 32 + l32];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bv[slot][ni] = Bs[buf][kk + lhi][wn0 + ni * 32 + l32];
    };

    // Software pipeline.  A depth tile is NSTEP MFMA steps of depth 2; each step
    // issues NMF MFMAs, and between consecutive MFMAs sits one "slot" of other
    // work, so that this work issues while the matrix pipe is busy:
    //   step 0     : registers holding tile t+1 go to the other LDS buffer; the
    //                table rows of tile t+2 are fetched (scalar)
    //   steps 1..4 : the global loads of tile t+2 are issued into those registers
    //   every step : operands of the next step are read from LDS first; the last
    //                step waits for its own operand reads, passes the workgroup
    //                barrier and reads the first operands of tile t+1, so barrier
    //                and LDS latency sit under that step's MFMAs.
    // The barrier orders LDS traffic only; global loads stay in flight across it.
    // Tile indices past the end are clamped (loading or storing a tile nobody
    // consumes is harmless), which keeps the loop free of branches.
    constexpr int NSTEP = BK / 2;
    constexpr int NMF = MI * NI;
    constexpr int GSLOTS = 4 * NMF;          // slots of steps 1..4
    const int ntiles = ph.depth_tiles;
    const int last = ntiles - 1;
    if (ntiles > 0) {
        table_fetch(0);
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i) gather_issue(i);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) filter_issue(0, i);
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i) store_b(0, i);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) store_a(0, i);
        const int t1 = last < 1 ? last : 1;
        table_fetch(t1);
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i) gather_issue(i);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) filter_issue(t1, i);
    }
    lds_barrier();
    if (ntiles > 0) read_ops(0, 0, 0);
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        const int t2 = (t + 2 < ntiles) ? t + 2 : last;
#pragma unroll
        for (int j = 0; j < NSTEP; ++j) {
            const int cur = j & 1, nxt = cur ^ 1;
            if (j + 1 < NSTEP) {
                read_ops(buf, 2 * (j + 1), nxt);
            } else {
                lds_barrier();
                read_ops(buf ^ 1, 0, nxt);
            }
            // all side work of the step first, then its MFMAs back to back: every
            // switch between the matrix pipe and other instructions costs a
            // pipeline drain, so one gap per step beats one per MFMA
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
                if (j == 0) {
#pragma unroll
                    for (int i = 0; i < B_ROWS; ++i)
                        if (i * NMF / B_ROWS == q) store_b(buf ^ 1, i);
                    if (q < A_PER_THREAD) store_a(buf ^ 1, q);
                    if (q == NMF - 1) table_fetch(t2);
                } else if (j <= 4) {
                    const int sidx = (j - 1) * NMF + q;
#pragma unroll
                    for (int i = 0; i < B_ROWS; ++i)
                        if (i * GSLOTS / B_ROWS == sidx) gather_issue(i);
                    if (sidx < A_PER_THREAD) filter_issue(t2, sidx);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NMF; ++q)
                acc[q / NI][q % NI] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                    av[cur][q / NI], bv[cur][q % NI], acc[q / NI][q % NI], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- epilogue: bias + store.  Accumulator element v of lane L is
    // row 8*(v/4) + 4*(L/32) + v%4, column L%32 of the 32x32 tile. ----
    float bz[MI][16];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = kt * BM + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
            bz[mi][v] = (a.bias && k < a.Kout) ? a.bias[k] : 0.f;
        }
    if (a.d2s_C > 0) {
        // depth-to-space store: GEMM row k' -> (pa, pb, c)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int m = pt * BN + wn0 + ni * 32 + l32;
            if (m >= Mpix) continue;
            const int n = m / HWs, rem = m - n * HWs;
            const int oh = rem / ph.Ws, ow = rem - oh * ph.Ws;
            const int h0 = oh * a.d2s_sh, v0 = ow * a.d2s_sw;
            float *op = a.out + (int64_t)n * a.out_img_stride + h0 * a.Wout + v0;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = kt * BM + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                    const int pab = (int)fast_div((uint32_t)k, a.div_d2s_C), c = k - pab * a.d2s_C;
                    const int pa = (int)fast_div((uint32_t)pab, a.div_d2s_sw), pb = pab - pa * a.d2s_sw;
                    if (k < a.Kout && h0 + pa < a.Hout && v0 + pb < a.Wout)
                        op[(int64_t)c * a.out_chan_stride + pa * a.Wout + pb] = acc[mi][ni][v];
                }
            }
        }
        return;
    }
    if (a.ngroup > 0) {
        // grouped outputs: GEMM row k is filter k - k0[g] of group g, stored to that
        // group's own tensor (forward only: stride-1 output walk, one phase)
        const int k1 = a.grp_k0[1], k2 = a.grp_k0[2], k3 = a.grp_k0[3];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int m = pt * BN + wn0 + ni * 32 + l32;
            if (m >= Mpix) continue;
            const int n = m / HWs, rem = m - n * HWs;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = kt * BM + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                    if (k >= a.Kout) continue;
                    const int g = (k >= k1) + (k >= k2) + (k >= k3);
                    float *o = g == 0 ? a.grp_out[0] : g == 1 ? a.grp_out[1] : g == 2 ? a.grp_out[2] : a.grp_out[3];
                    const float *bp = g == 0 ? a.grp_bias[0] : g == 1 ? a.grp_bias[1] : g == 2 ? a.grp_bias[2] : a.grp_bias[3];
                    const int k0 = g == 0 ? a.grp_k0[0] : g == 1 ? k1 : g == 2 ? k2 : k3;
                    const int kend = g == 0 ? k1 : g == 1 ? k2 : g == 2 ? k3 : a.grp_k0[4];
                    const int kl = k - k0, Kg = kend - k0;
                    o[((int64_t)n * Kg + kl) * a.out_chan_stride + rem] = acc[mi][ni][v] + (bp ? bp[kl] : 0.f);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int m = pt * BN + wn0 + ni * 32 + l32;
        if (m >= Mpix) continue;
        const int n = m / HWs, rem = m - n * HWs;
        const int oh = rem / ph.Ws, ow = rem - oh * ph.Ws;
        const int h = oh * a.out_step_h + ph.out_base_h;
        const int v_ = ow * a.out_step_w + ph.out_base_w;
        float *op = a.out + (int64_t)n * a.out_img_stride + h * a.Wout + v_;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * BM + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                float val = acc[mi][ni][v] + bz[mi][v];
                if (a.relu) val = fmaxf(val, 0.f);
                if (k < a.Kout) op[(int64_t)k * a.out_chan_stride] = val;
            }
        }
    }
}

static const int kFilterTile[4] = {128, 64, 32, 96};
static const int kPixelTile[4] = {128, 256, 256, 128};
int gemmconv_filter_tile(int tile) { return kFilterTile[tile]; }
int gemmconv_pixel_tile(int tile) { return kPixelTile[tile]; }

template <bool PW>
static void launch_gemmconv_t(const GemmConvArgs &a, int tile, dim3 grid, hipStream_t s)
{
    switch (tile) {
    case 0:
        hipLaunchKernelGGL((gemmconv_kernel<128, 128, 64, 64, PW>), grid, dim3(256), 0, s, a);
        break;
    case 1:
        hipLaunchKernelGGL((gemmconv_kernel<64, 256, 64, 64, PW>), grid, dim3(256), 0, s, a);
        break;
    case 2:
        hipLaunchKernelGGL((gemmconv_kernel<32, 256, 32, 64, PW>), grid, dim3(256), 0, s, a);
        break;
    default:    // 96 filters: three 32-row MFMA tiles per wave (filter counts 96, 192, ...)
        hipLaunchKernelGGL((gemmconv_kernel<96, 128, 96, 32, PW>), grid, dim3(256), 0, s, a);
        break;
    }
}

hipError_t launch_gemmconv(const GemmConvArgs &a, int tile, int nphases, hipStream_t s)
{
    const dim3 grid((unsigned)(a.tiles_k * a.tiles_pix), (unsigned)nphases);
    if (a.pw_depth > 0) launch_gemmconv_t<true>(a, tile, grid, s);
    else launch_gemmconv_t<false>(a, tile, grid, s);
    return hipGetLastError();
}

}  // namespace mi355conv
