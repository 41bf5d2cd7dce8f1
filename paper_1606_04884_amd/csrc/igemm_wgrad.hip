// Backward-weight implicit GEMM on fp32 MFMA for gfx950, plus the reductions
// across the batch (split partial sums, bias gradient).
//
// dw[k][j] = sum_m dy[m][k] * lowered(x)[m][j],  m = (n,p,q),  j = (c,r,s).
// Sec. 4.2 "im2col" of the paper notes that per-image products are small and
// that lowering many images into one product is what pays; here the batch and
// the output pixels together form the reduction axis of ONE product, which is
// cut into `splits` ranges so that a small filter gradient (e.g. 64 x 576)
// still fills 256 compute units.  Every workgroup reduces its range in
// registers and writes a partial tile; split_reduce_kernel adds the partials in
// a fixed order (deterministic, no atomics).
//
// Filters k are the MFMA "A" rows and lowered columns j the "B" columns, so the
// 32 lanes of a half-wave hold 32 consecutive (c,r,s) of one filter: KCRS stores
// are contiguous.  Both operands are read with lanes along the pixel axis (the
// contiguous axis of dy and x) and written to LDS transposed, with an odd row
// pitch so that neither the transposed writes nor the MFMA operand reads
// conflict.

#include "conv_internal.h"

namespace mi355conv {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int xcd_remap_w(int id, int nb)
{
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = id & 7, local = id >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}

// Workgroup barrier that orders LDS traffic only (global loads stay in flight).
__device__ __forceinline__ void lds_barrier_w()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void wgrad_kernel(WgradArgs a)
{
    constexpr int BK = 32;                   // pixels per main-loop step
    constexpr int WAVES_N = BN / WN;
    constexpr int WAVES_MN = (BM / WM) * WAVES_N;     // waves tiling the output tile
    constexpr int WAVES_K = 4 / WAVES_MN;             // waves sharing one output sub-tile: each
    static_assert(WAVES_MN * WAVES_K == 4, "4 waves per workgroup");   // takes a slice of every step
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int A_PER_THREAD = BM / 8;     // 8 thread rows x 32 pixels
    constexpr int B_PER_THREAD = BN / 8;

    __shared__ float As[2][BK][BM + 1];
    __shared__ float Bs[2][BK][BN + 1];
    __shared__ int2 coltab[BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int ntile = a.tiles_k * a.tiles_j;
    const int logical = xcd_remap_w(blockIdx.x, gridDim.x);
    const int tile_id = logical % ntile;     // tiles of one split are neighbours
    const int split = logical / ntile;
    const int kt = tile_id % a.tiles_k;
    const int jt = tile_id / a.tiles_k;

    // column table: lowered column j -> element offset and tap (r, t)
    if (tid < BN) {
        const int j = jt * BN + tid;
        int2 e;
        e.x = 0;
        e.y = kInvalidDr << 16;
        if (j < a.CRS) {
            const int c = (int)fast_div((uint32_t)j, a.div_RS);
            const int rt = j - c * a.R * a.S;
            const int r = (int)fast_div((uint32_t)rt, a.div_S);
            const int t = rt - r * a.S;
            e.x = c * a.H * a.W + r * a.W + t;
            e.y = (r << 16) | t;
        }
        coltab[tid] = e;
    }
    __syncthreads();

    const int pp = tid & 31;       // pixel within the step
    const int trow = tid >> 5;     // 0..7: first filter / column handled
    const int m_begin = split * a.chunk;
    const int m_end = min(a.M, m_begin + a.chunk);
    const int nsteps = (m_end - m_begin + BK - 1) / BK;

    float areg[A_PER_THREAD], breg[B_PER_THREAD];
    uint32_t amask = 0, bmask = 0;   // validity bits, applied when the values reach LDS
    int2 col[B_PER_THREAD];          // this thread's lowered columns, fixed for the whole kernel
#pragma unroll
    for (int i = 0; i < B_PER_THREAD; ++i) col[i] = coltab[trow + i * 8];

    // per-step pixel state of the tile being loaded
    bool pv = false;
    int dy_base = 0, x_base = 0, ih0 = 0, iw0 = 0;
    auto pixel_setup = [&](int step) {
        const int m = m_begin + step * BK + pp;
        pv = m < m_end;
        const int mm = pv ? m : 0;
        const int n = (int)fast_div((uint32_t)mm, a.div_PQ);
        const int pq = mm - n * a.PQ;
        const int p = (int)fast_div((uint32_t)pq, a.div_Q);
        const int q = pq - p * a.Q;
        dy_base = n * a.K * a.PQ + pq;                   // dy[n][k][pq]
        const int ih_true = p * a.stride_h - a.pad_h;
        ih0 = pv ? ih_true : -(1 << 24);                 // a row no tap can bring in range
        iw0 = q * a.stride_w - a.pad_w;
        x_base = n * a.C * a.H * a.W + ih_true * a.W + iw0;
    };
    auto load_a = [&](int i) {
        const int k = kt * BM + trow + i * 8;
        const bool ok = pv && k < a.K;
        areg[i] = a.dy[ok ? dy_base + k * a.PQ : 0];
        amask = (amask & ~(1u << i)) | (ok ? (1u << i) : 0u);
    };
    auto load_b = [&](int i) {
        const int2 e = col[i];
        const int r = e.y >> 16, t = e.y & 0xffff;
        const bool ok = ((unsigned)(ih0 + r) < (unsigned)a.H) && ((unsigned)(iw0 + t) < (unsigned)a.W);
        breg[i] = a.x[ok ? x_base + e.x : 0];
        bmask = (bmask & ~(1u << i)) | (ok ? (1u << i) : 0u);
    };
    float bsum[A_PER_THREAD];        // running sums of dy per filter (bias gradient)
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) bsum[i] = 0.f;
    auto store_a = [&](int buf, int i) {
        const float v = ((amask >> i) & 1u) ? areg[i] : 0.f;
        As[buf][pp][trow + i * 8] = v;
        bsum[i] += v;                // every pixel of the range passes here exactly once
    };
    auto store_b = [&](int buf, int i) {
        Bs[buf][pp][trow + i * 8] = ((bmask >> i) & 1u) ? breg[i] : 0.f;
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    const int wave_mn = wave % WAVES_MN, wave_k = wave / WAVES_MN;
    const int wm0 = (wave_mn / WAVES_N) * WM;
    const int wn0 = (wave_mn % WAVES_N) * WN;
    const int l32 = lane & 31, lhi = lane >> 5;

    float av[2][MI], bv[2][NI];
    auto read_ops = [&](int buf, int kk, int slot) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) av[slot][mi] = As[buf][kk + lhi][wm0 + mi * 32 + l32];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bv[slot][ni] = Bs[buf][kk + lhi][wn0 + ni * 32 + l32];
    };

    // Software pipeline, same shape as the gather kernel's: per 32-pixel tile a
    // wave runs NSTEPW MFMA steps (its slice of the tile's 16 depth-2 steps) of
    // NMF MFMAs; between consecutive MFMAs sits one slot of other work:
    //   first eighth of the slots : registers holding tile t+1 go to the other LDS buffer
    //   next slot                 : pixel coordinates of tile t+2
    //   following half            : global loads of tile t+2
    //   last step                 : LDS-only barrier, then the first operands of tile t+1
    constexpr int NSTEP = BK / 2;
    constexpr int NSTEPW = NSTEP / WAVES_K;
    constexpr int NMF = MI * NI;
    constexpr int NSLOT = NSTEPW * NMF;
    constexpr int NEL = A_PER_THREAD + B_PER_THREAD;
    constexpr int SSLOTS = NSLOT / 8 > 0 ? NSLOT / 8 : 1;
    constexpr int LSLOTS = NSLOT / 2;
    static_assert(SSLOTS + 1 + LSLOTS <= NSLOT - NMF, "side work must end before the barrier step");
    auto load_el = [&](int e) { if (e < A_PER_THREAD) load_a(e); else load_b(e - A_PER_THREAD); };
    auto store_el = [&](int buf, int e) { if (e < A_PER_THREAD) store_a(buf, e); else store_b(buf, e - A_PER_THREAD); };
    const int kk0 = wave_k * NSTEPW * 2;     // first depth index of this wave's slice

    if (nsteps > 0) {
        pixel_setup(0);
#pragma unroll
        for (int e = 0; e < NEL; ++e) load_el(e);
#pragma unroll
        for (int e = 0; e < NEL; ++e) store_el(0, e);
        pixel_setup(1);          // past the end: every element masked off
#pragma unroll
        for (int e = 0; e < NEL; ++e) load_el(e);
    }
    lds_barrier_w();
    if (nsteps > 0) read_ops(0, kk0, 0);
    for (int st = 0; st < nsteps; ++st) {
        const int buf = st & 1;
#pragma unroll
        for (int j = 0; j < NSTEPW; ++j) {
            const int cur = j & 1, nxt = cur ^ 1;
            if (j + 1 < NSTEPW) {
                read_ops(buf, kk0 + 2 * (j + 1), nxt);
            } else {
                lds_barrier_w();
                read_ops(buf ^ 1, kk0, nxt);
            }
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
                const int sidx = j * NMF + q;
                if (sidx < SSLOTS) {
#pragma unroll
                    for (int e = 0; e < NEL; ++e)
                        if (e * SSLOTS / NEL == sidx) store_el(buf ^ 1, e);
                } else if (sidx == SSLOTS) {
                    pixel_setup(st + 2);
                } else if (sidx <= SSLOTS + LSLOTS) {
                    const int l = sidx - SSLOTS - 1;
#pragma unroll
                    for (int e = 0; e < NEL; ++e)
                        if (e * LSLOTS / NEL == l) load_el(e);
                }
            }
            // the step's MFMAs back to back (one switch between the matrix pipe and
            // other instructions per step instead of one per MFMA)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NMF; ++q)
                acc[q / NI][q % NI] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                    av[cur][q / NI], bv[cur][q % NI], acc[q / NI][q % NI], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // bias gradient: the workgroups of column tile 0 reduce their sums over the 32
    // pixel lanes and write one partial per (split, filter)
    if (a.bias_part != nullptr && jt == 0) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            float v = bsum[i];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 16);
            const int k = kt * BM + trow + i * 8;
            if (pp == 0 && k < a.K) a.bias_part[split * a.K + k] = v;
        }
    }

    // waves that shared an output sub-tile add their accumulators through LDS
    if (WAVES_K > 1) {
        float *scratch = &As[0][0][0];
        static_assert((WAVES_K - 1) * WAVES_MN * MI * NI * 16 * 64 <= 2 * BK * (BM + 1), "scratch fits in As");
        __syncthreads();
        if (wave_k > 0) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        scratch[((((wave_k - 1) * WAVES_MN + wave_mn) * MI * NI + mi * NI + ni) * 16 + v) * 64 + lane] =
                            acc[mi][ni][v];
        }
        __syncthreads();
        if (wave_k > 0) return;
#pragma unroll
        for (int wk = 1; wk < WAVES_K; ++wk)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[mi][ni][v] +=
                            scratch[((((wk - 1) * WAVES_MN + wave_mn) * MI * NI + mi * NI + ni) * 16 + v) * 64 + lane];
    }

    // partial tile -> part[split][k][j]
    float *out = a.part + (int64_t)split * a.K * a.CRS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int j = jt * BN + wn0 + ni * 32 + l32;
        if (j >= a.CRS) continue;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * BM + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                if (k < a.K) out[(int64_t)k * a.CRS + j] = acc[mi][ni][v];
            }
    }
}

static const int kWFilterTile[4] = {128, 64, 32, 64};
static const int kWColTile[4] = {128, 128, 128, 32};
int wgrad_filter_tile(int tile) { return kWFilterTile[tile]; }
int wgrad_col_tile(int tile) { return kWColTile[tile]; }

hipError_t launch_wgrad(const WgradArgs &a, int tile, hipStream_t s)
{
    const dim3 grid((unsigned)(a.tiles_k * a.tiles_j * a.splits));
    const ProfScope ps(KID_WGRAD, 2.0 * a.M * (double)a.K * a.CRS,
                       4.0 * ((double)a.N * a.C * a.H * a.W + (double)a.M * a.K + (double)a.K * a.CRS), s);
    switch (tile) {
    case 0:
        hipLaunchKernelGGL((wgrad_kernel<128, 128, 64, 64>), grid, dim3(256), 0, s, a);
        break;
    case 1:
        hipLaunchKernelGGL((wgrad_kernel<64, 128, 32, 64>), grid, dim3(256), 0, s, a);
        break;
    case 2:
        hipLaunchKernelGGL((wgrad_kernel<32, 128, 32, 32>), grid, dim3(256), 0, s, a);
        break;
    default:    // narrow lowered matrix (first layers with 3x3 filters): two waves per sub-tile
        hipLaunchKernelGGL((wgrad_kernel<64, 32, 32, 32>), grid, dim3(256), 0, s, a);
        break;
    }
    return hipGetLastError();
}

// Bias gradient, final stage: db[k] = scale * sum of the per-split partial sums.  One wave
// per filter: lane l adds the partials l, l+64, ... in order, then the 64 lane sums are
// combined in a fixed butterfly order (deterministic).  It rides along with the reduction of
// the filter gradient as extra workgroups of the same launch (wave index = filter).
__device__ __forceinline__ void bias_final_wave(const BiasJob &b, int k, float scale)
{
    if (k >= b.K) return;
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    for (int i = lane; i < b.nsplit; i += 64) s += b.part[i * b.K + k];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m);
    s *= scale;
    if (lane == 0) b.db[k] = b.accumulate ? b.db[k] + s : s;
}

// dst[i] = scale * (sum over splits of part[s][i]) (+ dst[i]).  Eight interleaved
// partial sums (split s goes to sum s % 8) combined pairwise: a fixed order, so the
// result is reproducible, with eight loads in flight per thread.  Workgroups
// main_blocks.. do the bias job.
__global__ __launch_bounds__(256) void split_reduce_kernel(const float *__restrict__ part,
                                                           float *__restrict__ dst, int64_t count,
                                                           int splits, float scale, int accumulate,
                                                           int main_blocks, BiasJob bj)
{
    if ((int)blockIdx.x >= main_blocks) {
        bias_final_wave(bj, ((int)blockIdx.x - main_blocks) * 4 + (threadIdx.x >> 6), scale);
        return;
    }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)main_blocks * blockDim.x) {
        float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const float *p = part + i;
        int k = 0;
        for (; k + 8 <= splits; k += 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u) s[u] += p[(int64_t)(k + u) * count];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k + u < splits) s[u] += p[(int64_t)(k + u) * count];
        float t = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
        t *= scale;
        dst[i] = accumulate ? dst[i] + t : t;
    }
}

// The same sum for many splits of a small tensor, where one thread per element would
// leave most of the chip idle behind long chains of loads: 64 consecutive elements per
// workgroup, each of its eight waves adds an eighth of the splits (sixteen interleaved
// sums, combined pairwise), and wave 0 combines the eight results in a fixed order.
__global__ __launch_bounds__(512) void split_reduce_wide_kernel(const float *__restrict__ part,
                                                                float *__restrict__ dst, int64_t count,
                                                                int splits, float scale, int accumulate,
                                                                int main_blocks, BiasJob bj)
{
    __shared__ float sm[7][64];
    if ((int)blockIdx.x >= main_blocks) {
        bias_final_wave(bj, ((int)blockIdx.x - main_blocks) * 8 + (threadIdx.x >> 6), scale);
        return;
    }
    const int e = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + e;
    const int per = (splits + 7) / 8;
    const int k0 = q * per, k1 = min(splits, k0 + per);
    float s[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) s[u] = 0.f;
    if (i < count) {
        const float *p = part + i;
        int k = k0;
        for (; k + 16 <= k1; k += 16) {
#pragma unroll
            for (int u = 0; u < 16; ++u) s[u] += p[(int64_t)(k + u) * count];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (k + u < k1) s[u] += p[(int64_t)(k + u) * count];
    }
#pragma unroll
    for (int w = 8; w >= 1; w >>= 1)
#pragma unroll
        for (int u = 0; u < w; ++u) s[u] += s[u + w];
    if (q > 0) sm[q - 1][e] = s[0];
    __syncthreads();
    if (q == 0 && i < count) {
        float t = ((s[0] + sm[0][e]) + (sm[1][e] + sm[2][e])) + ((sm[3][e] + sm[4][e]) + (sm[5][e] + sm[6][e]));
        t *= scale;
        dst[i] = accumulate ? dst[i] + t : t;
    }
}

hipError_t launch_split_reduce(const float *part, float *dst, int64_t count, int splits,
                               float scale, int accumulate, const BiasJob &bj, hipStream_t s)
{
    const bool bias = bj.part != nullptr && bj.db != nullptr;
    if (splits >= 32 && count <= 256 * 1024) {
        const int main_blocks = (int)((count + 63) / 64);
        const int extra = bias ? (bj.K + 7) / 8 : 0;
        hipLaunchKernelGGL(split_reduce_wide_kernel, dim3((unsigned)(main_blocks + extra)), dim3(512), 0, s,
                           part, dst, count, splits, scale, accumulate, main_blocks, bj);
        return hipGetLastError();
    }
    int64_t blocks = (count + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    const int extra = bias ? (bj.K + 3) / 4 : 0;
    hipLaunchKernelGGL(split_reduce_kernel, dim3((unsigned)(blocks + extra)), dim3(256), 0, s, part, dst,
                       count, splits, scale, accumulate, (int)blocks, bj);
    return hipGetLastError();
}

// The same reduction for a filter gradient computed as 3x3 sub-filter gradients
// (Winograd backward-weight of filters larger than 3x3): element (k, c, r, s) of dw
// comes from part[split][k][q*C + c][(r % 3) * 3 + s % 3], q = (r / 3) * ceil(S / 3) + s / 3.
__global__ __launch_bounds__(256) void split_reduce_sub_kernel(const float *__restrict__ part,
                                                               float *__restrict__ dw, int K, int C,
                                                               int R, int S, int splits, float scale,
                                                               int accumulate, int main_blocks, BiasJob bj)
{
    if ((int)blockIdx.x >= main_blocks) {
        bias_final_wave(bj, ((int)blockIdx.x - main_blocks) * 4 + (threadIdx.x >> 6), scale);
        return;
    }
    const int nsw = (S + 2) / 3, nsub = ((R + 2) / 3) * nsw;
    const int64_t count = (int64_t)K * C * R * S;
    const int64_t src_count = (int64_t)K * nsub * C * 9;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)main_blocks * blockDim.x) {
        const int ss = (int)(i % S), r = (int)((i / S) % R);
        const int c = (int)((i / ((int64_t)R * S)) % C), k = (int)(i / ((int64_t)R * S * C));
        const int q = (r / 3) * nsw + ss / 3;
        const float *p = part + ((int64_t)k * nsub * C + (int64_t)q * C + c) * 9 + (r % 3) * 3 + ss % 3;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int j = 0;
        for (; j + 8 <= splits; j += 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u) acc[u] += p[(int64_t)(j + u) * src_count];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (j + u < splits) acc[u] += p[(int64_t)(j + u) * src_count];
        float t = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
        t *= scale;
        dw[i] = accumulate ? dw[i] + t : t;
    }
}

hipError_t launch_split_reduce_sub(const float *part, float *dw, int K, int C, int R, int S, int splits,
                                   float scale, int accumulate, const BiasJob &bj, hipStream_t s)
{
    const bool bias = bj.part != nullptr && bj.db != nullptr;
    int64_t blocks = ((int64_t)K * C * R * S + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    const int extra = bias ? (bj.K + 3) / 4 : 0;
    hipLaunchKernelGGL(split_reduce_sub_kernel, dim3((unsigned)(blocks + extra)), dim3(256), 0, s, part, dw, K,
                       C, R, S, splits, scale, accumulate, (int)blocks, bj);
    return hipGetLastError();
}

}  // namespace mi355conv
