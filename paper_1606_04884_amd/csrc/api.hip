// C-ABI entry points of libmi355conv: argument checks, algorithm choice,
// workspace layout and kernel launches.  See include/mi355conv.h for the contract.

#include "../../include/mi355conv.h"
#include "conv_internal.h"

#include <atomic>
#include <cstdlib>

using namespace mi355conv;

// Workspace of conv2d_fwd_static: one copy per GPU, loaded with this code object and held
// until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns (static_scratch()).
static __device__ __align__(256) unsigned char scratch[CONV2D_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device; two
// threads racing on the first call store the same value).  nullptr + *rc on failure.
void *static_scratch(int *rc)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *rc = CONV2D_ERR_LAUNCH;
        return nullptr;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            *rc = CONV2D_ERR_LAUNCH;
            return nullptr;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *rc = CONV2D_OK;
    return p;
}

constexpr int32_t kMaxDim = 16383;          // tap displacements are packed in 16 bits
constexpr int64_t kMaxElems = (int64_t(1) << 31) - 1;

struct Geom {
    int32_t N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
};

int check_desc(const conv2d_desc *d, Geom *g)
{
    if (!d) return CONV2D_ERR_NULL;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1)
        return CONV2D_ERR_GEOMETRY;
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return CONV2D_ERR_GEOMETRY;
    if (d->H > kMaxDim || d->W > kMaxDim || d->R > kMaxDim || d->S > kMaxDim ||
        d->pad_h > kMaxDim || d->pad_w > kMaxDim || d->stride_h > kMaxDim || d->stride_w > kMaxDim)
        return CONV2D_ERR_GEOMETRY;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return CONV2D_ERR_GEOMETRY;
    g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->K = d->K; g->R = d->R; g->S = d->S;
    g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    g->Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    if (g->P > kMaxDim || g->Q > kMaxDim) return CONV2D_ERR_GEOMETRY;
    const int64_t nx = (int64_t)g->N * g->C * g->H * g->W;
    const int64_t ny = (int64_t)g->N * g->K * g->P * g->Q;
    const int64_t nw = (int64_t)g->K * g->C * g->R * g->S;
    if (nx > kMaxElems || ny > kMaxElems || nw > kMaxElems) return CONV2D_ERR_GEOMETRY;
    // padded pixel counts are also held in 32 bits
    if ((int64_t)g->N * g->P * g->Q > kMaxElems - 512 || (int64_t)g->N * g->H * g->W > kMaxElems - 512)
        return CONV2D_ERR_GEOMETRY;
    return CONV2D_OK;
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }
int round_up(int a, int b) { return ceil_div(a, b) * b; }

// Tile choice of the gather kernel from a small cost model: a workgroup's depth
// step costs 64 issue cycles per MFMA plus ~4.3 per other instruction (measured:
// other instructions barely overlap MFMAs, not even those of another wave on the
// same SIMD, so co-resident workgroups share a compute unit's time rather than
// multiply its throughput), i.e. about 2600 / 3050 / 1950 / 2200 cycles for the
// 128x128 / 64x256 / 32x256 / 96x128 tiles; the busiest of the 256 compute units
// executes ceil(blocks / 256) workgroups.
int pick_gather_tile(int filters, int64_t pixels)
{
    static const double step_cycles[4] = {2608.0, 3040.0, 1970.0, 2180.0};
    int best = 0;
    double best_cost = 1e300;
    for (int t = 0; t < 4; ++t) {
        const int64_t blocks = (int64_t)ceil_div(filters, gemmconv_filter_tile(t)) *
                               ((pixels + gemmconv_pixel_tile(t) - 1) / gemmconv_pixel_tile(t));
        const double cost = (double)((blocks + 255) / 256) * step_cycles[t];
        if (cost < best_cost) { best_cost = cost; best = t; }
    }
    return best;
}

int pick_wgrad_tile(int filters, int crs)
{
    if (crs <= 32) return 3;            // 64 filters x 32 lowered columns
    static const double handicap[3] = {1.0, 1.03, 1.10};
    int best = 0;
    double best_cost = 1e30;
    for (int t = 0; t < 3; ++t) {
        const double cost = round_up(filters, wgrad_filter_tile(t)) * handicap[t];
        if (cost < best_cost) { best_cost = cost; best = t; }
    }
    return best;
}

// ---- workspace plans -------------------------------------------------------
int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

struct GatherPlan {
    int d2s;                    // backward-data as one gather with depth-to-space rows
    int dr_min, nd_r, dt_min, nd_t;
    int tile, Kpad;             // Kpad: columns of the filter matrix
    int nphases;                // all phases (may exceed kMaxPhases: launched in groups)
    int64_t rows_total;         // padded rows over all phases
    size_t wt_bytes, tab_bytes, total_bytes;
};

struct PhaseGeom {
    int r0, nr, t0, nt, rows, rows_pad, in_base_h, in_base_w, a, b, Hs, Ws;
};

// phase (a, b) of backward-data: output pixels h = a + i*sh, v = b + j*sw
PhaseGeom bwd_phase(const Geom &g, int a, int b)
{
    PhaseGeom p;
    p.a = a; p.b = b;
    p.r0 = (a + g.ph) % g.sh;
    p.t0 = (b + g.pw) % g.sw;
    p.nr = p.r0 < g.R ? ceil_div(g.R - p.r0, g.sh) : 0;
    p.nt = p.t0 < g.S ? ceil_div(g.S - p.t0, g.sw) : 0;
    p.rows = g.K * p.nr * p.nt;
    p.rows_pad = round_up(p.rows, kDepthTile);
    p.in_base_h = (a + g.ph - p.r0) / g.sh;
    p.in_base_w = (b + g.pw - p.t0) / g.sw;
    p.Hs = a < g.H ? ceil_div(g.H - a, g.sh) : 0;
    p.Ws = b < g.W ? ceil_div(g.W - b, g.sw) : 0;
    return p;
}

GatherPlan plan_fwd(const Geom &g)
{
    GatherPlan p = {};
    p.tile = pick_gather_tile(g.K, (int64_t)g.N * g.P * g.Q);
    p.Kpad = round_up(g.K, gemmconv_filter_tile(p.tile));
    p.nphases = 1;
    p.rows_total = round_up(g.C * g.R * g.S, kDepthTile);
    p.wt_bytes = align_up((size_t)p.rows_total * p.Kpad * sizeof(float), 256);
    p.tab_bytes = align_up((size_t)p.rows_total * sizeof(DepthEntry), 256);
    p.total_bytes = p.wt_bytes + p.tab_bytes;
    return p;
}

GatherPlan plan_bwd_data(const Geom &g)
{
    GatherPlan p = {};
    // Strided layers with few input channels (first layers): instead of one
    // sub-convolution per phase with C (<< 32) GEMM rows each, compute the
    // stride_h*stride_w*C values of every stride x stride block of dx as the rows of
    // ONE stride-1 gather over the union of the phases' tap displacements.
    if (g.sh * g.sw > 1) {
        const int rows = g.sh * g.sw * g.C;
        p.dr_min = floor_div(g.ph - g.R + 1 + g.sh - 1, g.sh);          // ceil((ph-R+1)/sh)
        p.dt_min = floor_div(g.pw - g.S + 1 + g.sw - 1, g.sw);
        p.nd_r = floor_div(g.sh - 1 + g.ph, g.sh) - p.dr_min + 1;
        p.nd_t = floor_div(g.sw - 1 + g.pw, g.sw) - p.dt_min + 1;
        const int64_t block_pixels = (int64_t)g.N * ceil_div(g.H, g.sh) * ceil_div(g.W, g.sw);
        const int tile = pick_gather_tile(rows, block_pixels);
        const double cost_d2s = (double)round_up(rows, gemmconv_filter_tile(tile)) * p.nd_r * p.nd_t;
        const int ptile = pick_gather_tile(g.C, block_pixels);
        const double cost_phase = (double)round_up(g.C, gemmconv_filter_tile(ptile)) * g.R * g.S;
        if (rows <= 256 && cost_d2s < cost_phase) {
            p.d2s = 1;
            p.tile = tile;
            p.Kpad = round_up(rows, gemmconv_filter_tile(tile));
            p.nphases = 1;
            p.rows_total = round_up(g.K * p.nd_r * p.nd_t, kDepthTile);
            p.wt_bytes = align_up((size_t)p.rows_total * p.Kpad * sizeof(float), 256);
            p.tab_bytes = align_up((size_t)p.rows_total * sizeof(DepthEntry), 256);
            p.total_bytes = p.wt_bytes + p.tab_bytes;
            return p;
        }
    }
    p.tile = pick_gather_tile(g.C, (int64_t)g.N * ceil_div(g.H, g.sh) * ceil_div(g.W, g.sw));
    p.Kpad = round_up(g.C, gemmconv_filter_tile(p.tile));
    p.nphases = g.sh * g.sw;
    p.rows_total = 0;
    for (int a = 0; a < g.sh; ++a)
        for (int b = 0; b < g.sw; ++b) p.rows_total += bwd_phase(g, a, b).rows_pad;
    if (p.rows_total == 0) p.rows_total = kDepthTile;
    p.wt_bytes = align_up((size_t)p.rows_total * p.Kpad * sizeof(float), 256);
    p.tab_bytes = align_up((size_t)p.rows_total * sizeof(DepthEntry), 256);
    p.total_bytes = p.wt_bytes + p.tab_bytes;
    return p;
}

struct WgradPlan {
    int tile, tiles_k, tiles_j, splits, chunk, bias_splits;
    size_t part_bytes, bias_bytes, total_bytes;
};

WgradPlan plan_wgrad(const Geom &g)
{
    WgradPlan p;
    const int CRS = g.C * g.R * g.S;
    const int64_t M = (int64_t)g.N * g.P * g.Q;
    p.tile = pick_wgrad_tile(g.K, CRS);
    p.tiles_k = ceil_div(g.K, wgrad_filter_tile(p.tile));
    p.tiles_j = ceil_div(CRS, wgrad_col_tile(p.tile));
    const int tiles = p.tiles_k * p.tiles_j;
    // Choose the number of ranges the reduction axis is cut into.  All workgroups
    // take equally long and co-resident ones share a compute unit's time, so the
    // busiest of the 256 compute units runs ceil(blocks / 256) of them; more
    // splits also mean more partial tiles to write and a longer chain of adds in
    // the reduction kernel.  Minimise an estimate of the three.
    const double flops = 2.0 * (double)M * g.K * CRS;
    int64_t max_splits = (M + 255) / 256;            // at least 256 pixels of depth each
    if (max_splits > 4096) max_splits = 4096;
    if (max_splits < 1) max_splits = 1;
    int best = 1;
    double best_t = 1e300;
    for (int64_t sp = 1; sp <= max_splits; ++sp) {
        const double blocks = (double)tiles * sp;
        const double rounds = (double)((int64_t)((blocks + 255) / 256));
        const double eff = blocks / (rounds * 256.0);
        const double t_mfma = flops / (0.6 * 155e12) / eff;
        const double t_part = 2.0 * sp * g.K * (double)CRS * 4.0 / 3.0e12;
        const double t_chain = 0.1e-6 * sp;
        const double t = t_mfma + t_part + t_chain;
        if (t < best_t) { best_t = t; best = (int)sp; }
    }
    int64_t chunk = (M + best - 1) / best;
    chunk = (chunk + 31) / 32 * 32;
    p.chunk = (int)chunk;
    p.splits = (int)((M + chunk - 1) / chunk);
    p.bias_splits = p.splits;       // the main kernel also sums dy: one partial per split
    p.part_bytes = align_up((size_t)p.splits * g.K * CRS * sizeof(float), 256);
    p.bias_bytes = align_up((size_t)p.bias_splits * g.K * sizeof(float), 256);
    p.total_bytes = p.part_bytes + p.bias_bytes;
    return p;
}

// ---- Winograd F(2x2,3x3) ---------------------------------------------------
struct WinoPlan {
    int Cin, Kout, Cpad, Kpad, Hin, Win, Hout, Wout, pad_h, pad_w, TH, TW, T, tiles_t, tiles_k, mode, nsub;
    int grid;                   // persistent workgroups
    size_t u_bytes, total_bytes;
};

// The fused kernel handles stride-1 layers with 3x3 filters, and for forward /
// backward-data also filters up to 6x6 as a sum of 3x3 sub-filters of shifted
// inputs, whose reduction channels are a multiple of its 8-channel chunk and whose
// gathered tensor fits 32-bit byte offsets.  Backward-data is the forward kernel on
// dy with the rotated filter and pad' = R - 1 - pad.
bool wino_applicable(const Geom &g, conv2d_op op)
{
    if (g.sh != 1 || g.sw != 1) return false;
    if (op == CONV2D_BWD_WEIGHT) {
        if (g.R < 3 || g.S < 3 || g.R > 6 || g.S > 6 || g.ph > g.R - 1 || g.pw > g.S - 1) return false;
        // 64x64 output tiles handled as two halves of 32: C and K multiples of 32
        if (g.C % 32 != 0 || g.K % 32 != 0) return false;
        return (int64_t)g.N * g.C * g.H * g.W * 4 < (int64_t(1) << 31) &&
               (int64_t)g.N * g.K * g.P * g.Q * 4 < (int64_t(1) << 31);
    }
    if (g.R < 3 || g.S < 3 || g.R > 6 || g.S > 6) return false;
    if (g.ph > g.R - 1 || g.pw > g.S - 1) return false;
    const int cin = op == CONV2D_FWD ? g.C : g.K;
    // the reduction channels come in chunks of 8; only the tile-pair kernel (3x3, pad_w 1,
    // even width and tile row) also takes a ragged last chunk
    if (cin % wino_chan_chunk() != 0) {
        const int win = op == CONV2D_FWD ? g.W : g.Q, wout = op == CONV2D_FWD ? g.Q : g.W;
        const int pw = op == CONV2D_FWD ? g.pw : g.S - 1 - g.pw;
        if (!(g.R == 3 && g.S == 3 && pw == 1 && win % 2 == 0 && ceil_div(wout, 2) % 2 == 0)) return false;
    }
    const int64_t in_elems = op == CONV2D_FWD ? (int64_t)g.N * g.C * g.H * g.W
                                              : (int64_t)g.N * g.K * g.P * g.Q;
    return in_elems * 4 < (int64_t(1) << 31);   // buffer offsets: see winograd.hip
}

WinoPlan plan_wino(const Geom &g, conv2d_op op)
{
    WinoPlan p;
    const bool fwd = op == CONV2D_FWD;
    p.Cin = fwd ? g.C : g.K;
    p.Kout = fwd ? g.K : g.C;
    p.Hin = fwd ? g.H : g.P;
    p.Win = fwd ? g.W : g.Q;
    p.Hout = fwd ? g.P : g.H;
    p.Wout = fwd ? g.Q : g.W;
    p.pad_h = fwd ? g.ph : g.R - 1 - g.ph;
    p.pad_w = fwd ? g.pw : g.S - 1 - g.pw;
    p.nsub = ceil_div(g.R, 3) * ceil_div(g.S, 3);     // 3x3 sub-filters of the filter
    p.Cpad = p.nsub * round_up(p.Cin, wino_chan_chunk());   // (a ragged Cin only with nsub == 1)
    p.Kpad = round_up(p.Kout, wino_filter_tile());
    p.TH = ceil_div(p.Hout, 2);
    p.TW = ceil_div(p.Wout, 2);
    // pad_w 1, even width and an even number of tiles per row: tile-pair kernel
    p.mode = (p.nsub == 1 && p.pad_w == 1 && p.Win % 2 == 0 && p.TW % 2 == 0) ? 1 : 0;
    p.T = g.N * p.TH * p.TW;
    p.tiles_t = ceil_div(p.T, wino_tile_block());
    p.tiles_k = p.Kpad / wino_filter_tile();
    const int tiles = p.tiles_t * p.tiles_k;
    p.grid = tiles < 256 ? tiles : 256;          // one resident workgroup per compute unit
    p.u_bytes = align_up((size_t)16 * p.Cpad * p.Kpad * sizeof(float), 256);
    p.total_bytes = p.u_bytes + align_up((size_t)p.grid * 2 * wino_partial_slot_floats() * sizeof(float), 256);
    return p;
}

struct WinoWgradPlan {
    int TH, TW, T, tiles_k, tiles_c, splits, tiles_per_split, bias_splits, mode, nsub, tiles_c_sub;
    size_t part_bytes, bias_bytes, total_bytes;
};

WinoWgradPlan plan_wino_wgrad(const Geom &g)
{
    WinoWgradPlan p;
    p.TH = ceil_div(g.P, 2);
    p.TW = ceil_div(g.Q, 2);
    // pad_w 1 and an even width: tile pairs fetched with vector loads, the tile grid
    // taken with an even row width (one phantom tile per row when the true one is odd)
    p.mode = 0;
    p.nsub = ceil_div(g.R, 3) * ceil_div(g.S, 3);       // 3x3 sub-filters (per-element kernel only)
    if (p.nsub == 1 && g.pw == 1 && g.W % 2 == 0) {
        p.mode = (p.TW & 1) ? 2 : 1;
        p.TW = round_up(p.TW, 2);
    }
    p.T = g.N * p.TH * p.TW;
    p.tiles_k = ceil_div(g.K, wino_wgrad_tile());
    p.tiles_c_sub = ceil_div(g.C, wino_wgrad_tile());
    p.tiles_c = p.nsub * p.tiles_c_sub;
    const int tiles = p.tiles_k * p.tiles_c;
    const int step = wino_wgrad_step();
    // one workgroup per compute unit is resident: fill 256 slots a whole number of times
    const double slots = 256.0;
    int max_splits = ceil_div(p.T, 8 * step);       // at least 8 steps each
    if (max_splits > 2048) max_splits = 2048;
    if (max_splits < 1) max_splits = 1;
    const double flops = 32.0 * (double)p.T * g.K * g.C * p.nsub;
    int best = 1;
    double best_t = 1e300;
    for (int sp = 1; sp <= max_splits; ++sp) {
        const double blocks = (double)tiles * sp;
        const double rounds = (double)((int64_t)((blocks + slots - 1) / slots));
        const double eff = blocks / (rounds * slots);
        const double t = flops / (0.6 * 155e12) / eff + 2.0 * sp * g.K * (double)g.C * p.nsub * 36.0 / 3.0e12 + 0.1e-6 * sp;
        if (t < best_t) { best_t = t; best = sp; }
    }
    p.tiles_per_split = round_up(ceil_div(p.T, best), step);
    p.splits = ceil_div(p.T, p.tiles_per_split);
    p.bias_splits = p.splits;       // the main kernel also sums dy: one partial per split
    p.part_bytes = align_up((size_t)p.splits * g.K * g.C * p.nsub * 9 * sizeof(float), 256);
    p.bias_bytes = align_up((size_t)p.bias_splits * g.K * sizeof(float), 256);
    p.total_bytes = p.part_bytes + p.bias_bytes;
    return p;
}

int launch_status(hipError_t e) { return e == hipSuccess ? CONV2D_OK : CONV2D_ERR_LAUNCH; }

// the workspace contract: present, large enough, 256-byte aligned
bool ws_ok(const void *ws, size_t ws_bytes, size_t need) { return ws && ws_bytes >= need && ((uintptr_t)ws & 255) == 0; }

// ---- Winograd F(4x4,3x3), unfused (wino4.hip) --------------------------------
struct W4Plan {
    bool ok;
    int Cin, Kout, Hin, Win, Hout, Wout, pad_h, pad_w, TH, TW, T, Tpad, Kpad, chunks, csub, nsub, cfg, split, split_tiles;
    size_t u_bytes, v_bytes, m_bytes, slot_bytes, total_bytes;
};

W4Plan plan_wino4(const Geom &g, conv2d_op op)
{
    W4Plan p = {};
    if (op == CONV2D_BWD_WEIGHT) return p;
    if (g.R < 3 || g.S < 3 || g.R > 6 || g.S > 6 || g.sh != 1 || g.sw != 1 || g.ph > g.R - 1 || g.pw > g.S - 1) return p;
    const bool fwd = op == CONV2D_FWD;
    p.nsub = ceil_div(g.R, 3) * ceil_div(g.S, 3);
    p.Cin = fwd ? g.C : g.K;
    p.Kout = fwd ? g.K : g.C;
    p.Hin = fwd ? g.H : g.P;
    p.Win = fwd ? g.W : g.Q;
    p.Hout = fwd ? g.P : g.H;
    p.Wout = fwd ? g.Q : g.W;
    p.pad_h = fwd ? g.ph : g.R - 1 - g.ph;
    p.pad_w = fwd ? g.pw : g.S - 1 - g.pw;
    p.TH = ceil_div(p.Hout, 4);
    p.TW = ceil_div(p.Wout, 4);
    const int64_t T = (int64_t)g.N * p.TH * p.TW;
    if (T > (int64_t(1) << 24) || p.Kout > 65535) return p;
    p.T = (int)T;
    p.csub = ceil_div(p.Cin, 8);
    p.chunks = p.nsub * p.csub;
    // the workgroup tile that pads the product least (ties: the wider column tile)
    int64_t best = -1;
    for (int cfg = 0; cfg < 3; ++cfg) {
        const int64_t cost = (int64_t)round_up(p.Kout, wino4_tile_m(cfg)) * round_up(p.T, wino4_tile_n(cfg));
        if (best < 0 || cost < best) { best = cost; p.cfg = cfg; }
    }
    p.Kpad = round_up(p.Kout, wino4_tile_m(p.cfg));
    p.Tpad = round_up(p.T, wino4_tile_n(p.cfg));
    // 32-bit byte offsets inside one position's slice of each operand, and inside `in`
    if ((int64_t)p.chunks * 2 * p.Kpad * 16 >= (int64_t(1) << 31)) return p;
    if ((int64_t)p.chunks * 2 * p.Tpad * 16 >= (int64_t(1) << 31)) return p;
    if ((int64_t)g.N * p.Cin * p.Hin * p.Win * 4 >= (int64_t(1) << 31)) return p;
    p.u_bytes = align_up((size_t)36 * p.chunks * 8 * p.Kpad * sizeof(float), 256);
    p.v_bytes = align_up((size_t)36 * p.chunks * 8 * p.Tpad * sizeof(float), 256);
    p.m_bytes = align_up((size_t)36 * p.Kpad * p.Tpad * sizeof(float), 256);
    // 512 workgroups are resident (two per compute unit) and all take equally long, so the
    // GEMM runs in rounds; the tiles of the last, partly filled round are cut into `split`
    // equal depth shares when that fills the round(s) better.  Cost of a share in chunk
    // times: its chunks plus ~4 for start-up and the store of the partial tile.
    const int64_t tiles = (int64_t)36 * (p.Kpad / wino4_tile_m(p.cfg)) * (p.Tpad / wino4_tile_n(p.cfg));
    if (tiles >= (int64_t(1) << 24)) return p;
    const int rem = (int)(tiles % 512);
    p.split = 1;
    p.split_tiles = 0;
    if (rem > 0) {
        double best_t = (double)p.chunks + 4.0;           // one more round of whole tiles
        for (int sp = 2; sp <= 8 && sp <= p.chunks && rem * sp <= 1024; ++sp) {
            const double t = (double)ceil_div(rem * sp, 512) * ((double)ceil_div(p.chunks, sp) + 4.0) + 2.0;
            if (t < best_t) { best_t = t; p.split = sp; }
        }
        if (p.split > 1) p.split_tiles = rem;
    }
    p.slot_bytes = align_up((size_t)p.split_tiles * p.split * wino4_tile_m(p.cfg) * wino4_tile_n(p.cfg) * sizeof(float), 256);
    p.total_bytes = p.u_bytes + p.v_bytes + p.m_bytes + p.slot_bytes;
    p.ok = true;
    return p;
}

int run_wino4(const Geom &g, conv2d_op op, const float *in, const float *w, const float *bias, float *out,
              void *ws, size_t ws_bytes, hipStream_t s, int relu = 0)
{
    const W4Plan p = plan_wino4(g, op);
    if (!p.ok) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    W4Args a = {};
    a.in = in; a.w = w; a.bias = bias; a.out = out; a.relu = relu;
    a.U = (float *)ws;
    a.V = (float *)((char *)ws + p.u_bytes);
    a.M = (float *)((char *)ws + p.u_bytes + p.v_bytes);
    a.slots = (float *)((char *)ws + p.u_bytes + p.v_bytes + p.m_bytes);
    a.split = p.split; a.split_tiles = p.split_tiles;
    a.mode = op == CONV2D_FWD ? 0 : 1;
    a.C = g.C;
    a.N = g.N; a.Cin = p.Cin; a.Hin = p.Hin; a.Win = p.Win; a.Kout = p.Kout; a.Kpad = p.Kpad;
    a.Hout = p.Hout; a.Wout = p.Wout; a.pad_h = p.pad_h; a.pad_w = p.pad_w;
    a.TH = p.TH; a.TW = p.TW; a.T = p.T; a.Tpad = p.Tpad; a.chunks = p.chunks;
    a.R = g.R; a.S = g.S; a.csub = p.csub; a.nsw = ceil_div(g.S, 3);
    a.in_bytes = (int32_t)((int64_t)g.N * p.Cin * p.Hin * p.Win * 4);
    a.tile_cfg = p.cfg;
    return launch_status(launch_wino4(a, s));
}

struct W4WgradPlan {
    bool ok;
    int TH, TW, T, chunks, Kpad, Cpad, cfg, split, tiles, nsub;
    size_t wm_bytes, vm_bytes, slot_bytes, d_bytes, bias_bytes, total_bytes;
};

W4WgradPlan plan_wino4_wgrad(const Geom &g)
{
    W4WgradPlan p = {};
    if (g.R < 3 || g.S < 3 || g.R > 6 || g.S > 6 || g.sh != 1 || g.sw != 1 || g.ph > g.R - 1 || g.pw > g.S - 1) return p;
    p.nsub = ceil_div(g.R, 3) * ceil_div(g.S, 3);
    if ((int64_t)g.N * g.C * g.H * g.W * 4 >= (int64_t(1) << 31) || (int64_t)g.N * g.K * g.P * g.Q * 4 >= (int64_t(1) << 31))
        return p;
    p.TH = ceil_div(g.P, 4);
    p.TW = ceil_div(g.Q, 4);
    const int64_t T = (int64_t)g.N * p.TH * p.TW;
    if (T < 16 || T > 524000 || g.K > 65535) return p;        // the chunks are a grid dimension
    p.T = (int)T;
    p.chunks = ceil_div(p.T, 8);
    int64_t best = -1;
    for (int cfg = 0; cfg < 3; ++cfg) {
        const int64_t cost = (int64_t)round_up(g.K, wino4_tile_m(cfg)) * round_up(p.nsub * g.C, wino4_tile_n(cfg));
        if (best < 0 || cost < best) { best = cost; p.cfg = cfg; }
    }
    p.Kpad = round_up(g.K, wino4_tile_m(p.cfg));
    p.Cpad = round_up(p.nsub * g.C, wino4_tile_n(p.cfg));
    if ((int64_t)p.chunks * 2 * p.Kpad * 16 >= (int64_t(1) << 31) || (int64_t)p.chunks * 2 * p.Cpad * 16 >= (int64_t(1) << 31))
        return p;
    p.tiles = 36 * (p.Kpad / wino4_tile_m(p.cfg)) * (p.Cpad / wino4_tile_n(p.cfg));
    // depth shares per tile: fill the 512 resident workgroups a whole number of times; a
    // share costs its chunks plus ~4 chunk times of start-up and partial-tile store
    double best_t = 1e300;
    p.split = 2;
    for (int sp = 2; sp <= 64 && sp <= p.chunks && (int64_t)p.tiles * sp <= 2048; ++sp) {
        const double t = (double)ceil_div(p.tiles * sp, 512) * ((double)ceil_div(p.chunks, sp) + 4.0);
        if (t < best_t) { best_t = t; p.split = sp; }
    }
    if ((int64_t)p.tiles * p.split > 4096) return p;
    p.wm_bytes = align_up((size_t)36 * p.chunks * 8 * p.Kpad * sizeof(float), 256);
    p.vm_bytes = align_up((size_t)36 * p.chunks * 8 * p.Cpad * sizeof(float), 256);
    p.slot_bytes = align_up((size_t)p.tiles * p.split * wino4_tile_m(p.cfg) * wino4_tile_n(p.cfg) * sizeof(float), 256);
    p.d_bytes = align_up((size_t)36 * p.Kpad * p.Cpad * sizeof(float), 256);
    p.bias_bytes = align_up((size_t)p.chunks * 2 * p.Kpad * sizeof(float), 256);
    p.total_bytes = p.wm_bytes + p.vm_bytes + p.slot_bytes + p.d_bytes + p.bias_bytes;
    p.ok = true;
    return p;
}

int run_wino4_wgrad(const Geom &g, const float *x, const float *dy, float *dw, float *dbias, float scale,
                    int accumulate, void *ws, size_t ws_bytes, hipStream_t s)
{
    const W4WgradPlan p = plan_wino4_wgrad(g);
    if (!p.ok) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    W4WgradArgs a = {};
    a.x = x; a.dy = dy; a.dw = dw; a.db = dbias;
    a.Wm = (float *)ws;
    a.Vm = (float *)((char *)ws + p.wm_bytes);
    a.slots = (float *)((char *)ws + p.wm_bytes + p.vm_bytes);
    a.D = (float *)((char *)ws + p.wm_bytes + p.vm_bytes + p.slot_bytes);
    a.bias_part = dbias ? (float *)((char *)ws + p.wm_bytes + p.vm_bytes + p.slot_bytes + p.d_bytes) : nullptr;
    a.scale = scale; a.accumulate = accumulate;
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.P = g.P; a.Q = g.Q; a.pad_h = g.ph; a.pad_w = g.pw;
    a.TH = p.TH; a.TW = p.TW; a.T = p.T; a.chunks = p.chunks; a.Kpad = p.Kpad; a.Cpad = p.Cpad;
    a.R = g.R; a.S = g.S; a.nsub = p.nsub; a.nsw = ceil_div(g.S, 3);
    a.x_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    a.dy_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
    a.tile_cfg = p.cfg; a.split = p.split;
    a.div_THW = make_fastdiv((uint32_t)(p.TH * p.TW));
    a.div_TW = make_fastdiv((uint32_t)p.TW);
    return launch_status(launch_wino4_wgrad(a, s));
}

// the gather kernel's launch, timed when profiling is on (`share`: this launch's part of the pass)
int run_gemmconv(const GemmConvArgs &a, int tile, int nphases, const Geom &g, double share, hipStream_t s)
{
    const double flops = 2.0 * g.N * (double)g.K * g.P * g.Q * g.C * g.R * g.S * share;
    const double bytes = 4.0 * ((double)g.N * g.C * g.H * g.W + (double)g.N * g.K * g.P * g.Q + (double)g.K * g.C * g.R * g.S) * share;
    const ProfScope ps(KID_GEMMCONV, flops, bytes, s);
    return launch_status(launch_gemmconv(a, tile, nphases, s));
}

bool s2d_applicable(const Geom &g, conv2d_op op);     // strided layer as a stride-1 3x3 layer, below
bool tap_stream_ok(const Geom &g);                    // forward pass with the filter bank in LDS, below
bool tap_stream_bwd_ok(const Geom &g);                // the same for a stride-1 backward-data pass
constexpr int kTapBwdMinRows = 12;                 // below that the 32-row MFMA tiles are mostly empty

// ---- frequency-domain path (fft.hip): one 32 x 32 tile per image ---------------------------
struct FftPlan {
    bool ok;
    int rows, cols, depth;      // of the complex product per frequency
    int chunks, Mpad, Npad, cfg, split, split_tiles;
    size_t a_bytes, b_bytes, m_bytes, slot_bytes, total_bytes;
};

// per frequency a complex (rows x depth) . (depth x cols) product.  forward: rows = images,
// depth = channels, columns = filters; backward-data: columns = channels, depth = filters;
// backward-weight: rows = filters, depth = images, columns = channels.  The column side is
// stored in 2 x 2 block form (2 * cols real columns)
FftPlan plan_fft(const Geom &g, conv2d_op op)
{
    FftPlan p = {};
    if (g.sh != 1 || g.sw != 1 || g.H + 2 * g.ph > 32 || g.W + 2 * g.pw > 32 || g.P < 1 || g.Q < 1) return p;
    if ((int64_t)g.N * g.C * g.H * g.W * 4 >= (int64_t(1) << 31) || (int64_t)g.N * g.K * g.P * g.Q * 4 >= (int64_t(1) << 31) ||
        (int64_t)g.K * g.C * g.R * g.S * 4 >= (int64_t(1) << 31))
        return p;
    p.rows = op == CONV2D_BWD_WEIGHT ? g.K : g.N;
    p.depth = op == CONV2D_FWD ? g.C : op == CONV2D_BWD_DATA ? g.K : g.N;
    p.cols = op == CONV2D_FWD ? g.K : g.C;
    if (p.rows > 65535 || p.cols > 32767) return p;          // grid dimensions of the transform kernels
    p.chunks = ceil_div(p.depth, 4);
    if (p.chunks > 65535) return p;
    int64_t best = -1;
    for (int cfg = 0; cfg < 4; ++cfg) {          // (the fourth tile, 128 x 128, exists for this path only)
        const int64_t cost = (int64_t)round_up(p.rows, wino4_tile_m(cfg)) * round_up(2 * p.cols, wino4_tile_n(cfg));
        if (best < 0 || cost < best) { best = cost; p.cfg = cfg; }
    }
    p.Mpad = round_up(p.rows, wino4_tile_m(p.cfg));
    p.Npad = round_up(2 * p.cols, wino4_tile_n(p.cfg));
    // 32-bit byte offsets inside each operand (the chunk is the slowest index)
    if ((int64_t)p.chunks * 2 * kFftFreqs * p.Mpad * 16 >= (int64_t(1) << 31) ||
        (int64_t)p.chunks * 2 * kFftFreqs * p.Npad * 16 >= (int64_t(1) << 31))
        return p;
    const int64_t tiles = (int64_t)kFftFreqs * (p.Mpad / wino4_tile_m(p.cfg)) * (p.Npad / wino4_tile_n(p.cfg));
    if (tiles >= (int64_t(1) << 22)) return p;
    // the last, partly filled round of the resident workgroups (512 of four waves, 1024 of two)
    // as depth shares (as in plan_wino4)
    const int resident = p.cfg == 3 ? 1024 : 512;
    const int rem = (int)(tiles % resident);
    p.split = 1;
    p.split_tiles = 0;
    if (rem > 0) {
        double best_t = (double)p.chunks + 4.0;
        for (int sp = 2; sp <= 8 && sp <= p.chunks && rem * sp <= 2 * resident; ++sp) {
            const double t = (double)ceil_div(rem * sp, resident) * ((double)ceil_div(p.chunks, sp) + 4.0) + 2.0;
            if (t < best_t) { best_t = t; p.split = sp; }
        }
        if (p.split > 1) p.split_tiles = rem;
    }
    p.a_bytes = align_up((size_t)kFftFreqs * p.chunks * 8 * p.Mpad * sizeof(float), 256);
    p.b_bytes = align_up((size_t)kFftFreqs * p.chunks * 8 * p.Npad * sizeof(float), 256);
    p.m_bytes = align_up((size_t)kFftFreqs * p.Mpad * p.Npad * sizeof(float), 256);
    p.slot_bytes = align_up((size_t)p.split_tiles * p.split * wino4_tile_m(p.cfg) * wino4_tile_n(p.cfg) * sizeof(float), 256);
    p.total_bytes = p.a_bytes + p.b_bytes + p.m_bytes + p.slot_bytes;
    p.ok = true;
    return p;
}

int run_fft(const Geom &g, conv2d_op op, const float *in, const float *w, const float *bias, float *out,
            void *ws, size_t ws_bytes, hipStream_t s, int relu = 0)
{
    const FftPlan p = plan_fft(g, op);
    if (!p.ok || op == CONV2D_BWD_WEIGHT) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    const bool fwd = op == CONV2D_FWD;
    FftArgs a = {};
    a.in = in; a.w = w; a.bias = bias; a.out = out; a.relu = relu;
    a.A = (float *)ws;
    a.B = (float *)((char *)ws + p.a_bytes);
    a.M = (float *)((char *)ws + p.a_bytes + p.b_bytes);
    a.slots = (float *)((char *)ws + p.a_bytes + p.b_bytes + p.m_bytes);
    a.split = p.split; a.split_tiles = p.split_tiles; a.tile_cfg = p.cfg;
    a.mode = fwd ? 0 : 1;
    a.C = g.C; a.N = g.N;
    a.Cin = p.depth; a.Kout = p.cols;
    a.Hin = fwd ? g.H : g.P; a.Win = fwd ? g.W : g.Q;
    a.Hout = fwd ? g.P : g.H; a.Wout = fwd ? g.Q : g.W;
    a.in_off_h = fwd ? g.ph : 0; a.in_off_w = fwd ? g.pw : 0;
    a.out_off_h = fwd ? 0 : g.ph; a.out_off_w = fwd ? 0 : g.pw;
    a.R = g.R; a.S = g.S;
    a.chunks = p.chunks; a.Mpad = p.Mpad; a.Npad = p.Npad;
    a.in_bytes = (int32_t)((int64_t)g.N * a.Cin * a.Hin * a.Win * 4);
    a.w_bytes = (int32_t)((int64_t)g.K * g.C * g.R * g.S * 4);
    return launch_status(launch_fft_conv(a, s));
}

int run_fft_wgrad(const Geom &g, const float *x, const float *dy, float *dw, float *dbias, float scale, int accumulate,
                  void *ws, size_t ws_bytes, hipStream_t s)
{
    const FftPlan p = plan_fft(g, CONV2D_BWD_WEIGHT);
    if (!p.ok) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    FftWgradArgs a = {};
    a.x = x; a.dy = dy; a.dw = dw; a.db = dbias;
    a.A = (float *)ws;
    a.B = (float *)((char *)ws + p.a_bytes);
    a.M = (float *)((char *)ws + p.a_bytes + p.b_bytes);
    a.slots = (float *)((char *)ws + p.a_bytes + p.b_bytes + p.m_bytes);
    a.split = p.split; a.split_tiles = p.split_tiles; a.tile_cfg = p.cfg;
    a.scale = scale; a.accumulate = accumulate;
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.P = g.P; a.Q = g.Q; a.R = g.R; a.S = g.S;
    a.pad_h = g.ph; a.pad_w = g.pw;
    a.chunks = p.chunks; a.Mpad = p.Mpad; a.Npad = p.Npad;
    a.x_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    a.dy_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
    return launch_status(launch_fft_wgrad(a, s));
}

// Estimated time of the frequency-domain path, seconds; huge where it does not apply or is
// not worth trying (3x3 and smaller filters, a handful of channels).  Fitted to its kernels'
// measured times on the 5x5 layers of the AlexNet and Overfeat configurations: ~3.2 ns per
// transformed image or filter, ~4.4 ns per inverse, the GEMM at ~120 TFLOP/s over its padded
// size plus ~30 us for its short depth and the fix-up, ~5 us per launch.
double fft_estimate(const Geom &g, conv2d_op op)
{
    const FftPlan p = plan_fft(g, op);
    if (!p.ok || g.R * g.S < 16 || p.rows < 32 || p.cols < 32 || p.depth < 32) return 1e30;
    const double n_in = op == CONV2D_BWD_WEIGHT ? (double)g.N * (g.K + g.C) : (double)g.K * g.C + (double)g.N * p.depth;
    const double n_out = op == CONV2D_BWD_WEIGHT ? (double)g.K * g.C : (double)g.N * p.cols;
    const double gemm = 2.0 * kFftFreqs * p.Mpad * (double)p.Npad * p.chunks * 8.0 / 120e12 + 30e-6;
    return 3.2e-9 * n_in + 4.4e-9 * n_out + gemm + 15e-6;
}

int resolve_algo(const Geom &g, conv2d_op op, int algo)
{
    const bool s2d_ok = s2d_applicable(g, op);
    const bool wino_ok = wino_applicable(g, op) || s2d_ok;
    switch (algo) {
    case CONV2D_ALGO_AUTO: {
        // strided first layers (few channels, filter of 3 x 3 strides): rearranged into a
        // stride-1 3x3 layer over stride^2 * C channels, which Winograd takes
        // (backward passes only: forward through the gather kernel is as fast, without the
        // rearranged copy)
        if (s2d_ok)
            return (op != CONV2D_FWD && g.sh * g.sw * g.C <= 64) ? CONV2D_ALGO_WINOGRAD : CONV2D_ALGO_IGEMM;
        // Winograd pays once the 16 GEMMs are deep enough to amortise the transforms
        const int nsub_f = ceil_div(g.R, 3) * ceil_div(g.S, 3);
        const bool pays_f = 4 * nsub_f * 14 <= g.R * g.S * 10;
        if (op == CONV2D_BWD_WEIGHT) {
            if (!(wino_ok && pays_f)) return CONV2D_ALGO_IGEMM;
            // many channels and filters on a small map: the unfused F(4x4,3x3) form when its
            // estimate (36 GEMMs at ~140 TFLOP/s, the last round of workgroups charged half of what it
            // leaves empty, transforms at 4.3 / 4.9 TB/s over x + V and dy + W, the partial products
            // written and read once, ~25 us of small launches; within 5% of the measured times of the
            // VGG-16, AlexNet and Overfeat layers) beats the fused F(3x3,2x2) kernels' (~108 TFLOP/s
            // executed with vector loads, ~88 on odd tile rows, ~73 with per-element loads)
            const W4WgradPlan w4 = plan_wino4_wgrad(g);
            if (w4.ok && g.C >= 64 && g.K >= 64) {
                const WinoWgradPlan f2 = plan_wino_wgrad(g);
                const double t_f2 = 32.0 * f2.T * g.C * (double)g.K * f2.nsub / (f2.mode == 1 ? 108e12 : f2.mode == 2 ? 88e12 : 73e12);
                const double tile_b = 4.0 * wino4_tile_m(w4.cfg) * wino4_tile_n(w4.cfg);
                const double x_b = 4.0 * g.N * (double)g.C * g.H * g.W, dy_b = 4.0 * g.N * (double)g.K * g.P * g.Q;
                const double vm_b = 4.0 * 36.0 * w4.chunks * 8 * (double)w4.Cpad, wm_b = 4.0 * 36.0 * w4.chunks * 8 * (double)w4.Kpad;
                const double fill = (double)w4.tiles * w4.split / (512.0 * ceil_div(w4.tiles * w4.split, 512));
                double t_gemm = 72.0 * w4.chunks * 8.0 * w4.Kpad * w4.Cpad / (140e12 * (0.5 + 0.5 * fill));
                if (t_gemm < (vm_b + wm_b) / 3.5e12) t_gemm = (vm_b + wm_b) / 3.5e12;      // operands streamed from HBM
                const double t_w4 = t_gemm + (x_b + vm_b) / 4.3e12 + (dy_b + wm_b) / 4.9e12 +
                                    2.0 * w4.tiles * (double)w4.split * tile_b / 5e12 + 25e-6;
                // filters beyond 3x3 on maps of at most 32 x 32: the product of spectra, when its
                // estimate is clearly below both
                const double t_best = t_w4 < 0.95 * t_f2 ? t_w4 : t_f2;
                if (fft_estimate(g, op) < 0.92 * t_best) return CONV2D_ALGO_FFT;
                if (t_w4 < 0.95 * t_f2) return CONV2D_ALGO_WINOGRAD4;
            }
            return CONV2D_ALGO_WINOGRAD;
        }
        // backward-data into <= 4 channels: Winograd/GEMM rows would be almost empty;
        // a direct kernel takes it when its alignment conditions hold, else the GEMM
        if (op == CONV2D_BWD_DATA && g.C <= 4) return CONV2D_ALGO_IGEMM;
        // filters beyond 3x3 whose bank fits in LDS: streamed over dy (pointwise.hip, taps form)
        if (op == CONV2D_BWD_DATA && (g.R > 3 || g.S > 3) && g.C >= kTapBwdMinRows && tap_stream_bwd_ok(g))
            return CONV2D_ALGO_IGEMM;
        const int cin = op == CONV2D_FWD ? g.C : g.K;
        // larger filters: 16 multiplications per 2x2 outputs and 3x3 sub-filter against
        // R*S*4 direct ones; the sub-filters of 4x4 / 4x5 filters are mostly padding
        const int nsub = ceil_div(g.R, 3) * ceil_div(g.S, 3);
        const bool pays = 4 * nsub * 14 <= g.R * g.S * 10;
        // a first layer (a handful of channels into many filters) is bound by writing its
        // output.  Up to four channels the taps form of the streaming kernel does that best
        // (the filter bank in LDS, 16-byte stores); else the tile-pair Winograd kernel (one
        // chunk per tile) does it at a better rate than the gather kernel's two-tile pipeline
        if (op == CONV2D_FWD && g.C <= 4 && tap_stream_ok(g)) return CONV2D_ALGO_IGEMM;
        if (wino_ok && op == CONV2D_FWD && g.C <= 8 && g.K >= 32 && g.R == 3 && g.S == 3 && g.pw == 1 &&
            g.W % 2 == 0 && ceil_div(g.Q, 2) % 2 == 0)
            return CONV2D_ALGO_WINOGRAD;
        if (wino_ok && cin >= 32 && pays) {
            // 3x3 with many channels on a small map: the unfused F(4x4,3x3) path when its
            // estimate beats the fused F(2x2,3x3) kernels' (measured rates on this chip:
            // 36 GEMMs at ~125 TFLOP/s unless streaming V and M at 3.5 TB/s takes longer, input
            // transform at 4.8 TB/s over input + V (3.5 without the wide row loads), output transform
            // at 4.5 TB/s over M + output,
            // ~25 us of small launches; fused: ~105 TFLOP/s executed for the tile-pair kernel,
            // ~76 for the one-tile-per-lane kernel)
            const W4Plan w4 = plan_wino4(g, op);
            if (w4.ok && cin >= 64) {
                const WinoPlan f2 = plan_wino(g, op);
                const double t_f2 = 32.0 * f2.T * f2.Cin * (double)f2.nsub * f2.Kpad / (f2.mode != 0 ? 105e12 : 76e12);
                const double in_b = 4.0 * g.N * (double)w4.Cin * w4.Hin * w4.Win, out_b = 4.0 * g.N * (double)w4.Kout * w4.Hout * w4.Wout;
                const double v_b = 4.0 * 36.0 * w4.chunks * 8 * (double)w4.Tpad, m_b = 4.0 * 36.0 * w4.Kpad * (double)w4.Tpad;
                // (the GEMM runs in rounds of 512 workgroups: a small layer leaves most of a round empty)
                const int64_t tiles = (int64_t)36 * (w4.Kpad / wino4_tile_m(w4.cfg)) * (w4.Tpad / wino4_tile_n(w4.cfg));
                const int64_t pieces = tiles - w4.split_tiles + (int64_t)w4.split_tiles * w4.split;
                const double fill = (double)pieces / (512.0 * (double)((pieces + 511) / 512));
                double t_gemm = 72.0 * w4.Tpad * (w4.chunks * 8.0) * w4.Kpad / (135e12 * fill);
                if (t_gemm < (v_b + m_b) / 3.5e12) t_gemm = (v_b + m_b) / 3.5e12;          // operands streamed from HBM
                const double t_w4 = t_gemm + (in_b + v_b) / (w4.pad_w <= 1 ? 4.8e12 : 3.5e12) + (m_b + out_b) / 4.5e12 + 25e-6;
                const double t_best = t_w4 < 0.95 * t_f2 ? t_w4 : t_f2;
                if (fft_estimate(g, op) < 0.92 * t_best) return CONV2D_ALGO_FFT;
                if (t_w4 < 0.95 * t_f2) return CONV2D_ALGO_WINOGRAD4;
            }
            return CONV2D_ALGO_WINOGRAD;
        }
        // filters the Winograd forms do not take (7x7 and up at stride 1), many channels: the
        // product of spectra against the implicit GEMM at ~85 TFLOP/s over the direct flops
        if (fft_estimate(g, op) < 0.8 * (2.0 * g.N * (double)g.K * g.C * g.P * g.Q * g.R * g.S / 85e12)) return CONV2D_ALGO_FFT;
        return CONV2D_ALGO_IGEMM;
    }
    case CONV2D_ALGO_IGEMM: return CONV2D_ALGO_IGEMM;
    case CONV2D_ALGO_WINOGRAD: return wino_ok ? CONV2D_ALGO_WINOGRAD : CONV2D_ERR_ALGO;
    case CONV2D_ALGO_WINOGRAD4:
        return (op == CONV2D_BWD_WEIGHT ? plan_wino4_wgrad(g).ok : plan_wino4(g, op).ok) ? CONV2D_ALGO_WINOGRAD4
                                                                                       : CONV2D_ERR_ALGO;
    case CONV2D_ALGO_FFT: return plan_fft(g, op).ok ? CONV2D_ALGO_FFT : CONV2D_ERR_ALGO;
    default: return CONV2D_ERR_ALGO;
    }
}

// 1x1 stride-1 unpadded layer whose pixel rows can be fetched as aligned 16-byte vectors
bool pointwise_ok(const Geom &g, const float *in, int64_t in_elems)
{
    return g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 &&
           (g.H * g.W) % 4 == 0 && ((uintptr_t)in & 15) == 0 && in_elems * 4 < (int64_t(1) << 31);
}

// 1x1 stride-1 unpadded layer whose small operand (filters x channels) fits in LDS and
// whose streamed tensor fits 32-bit byte offsets: the streaming kernel of pointwise.hip
bool pw_stream_ok(const Geom &g, conv2d_op op)
{
    if (g.R != 1 || g.S != 1 || g.sh != 1 || g.sw != 1 || g.ph != 0 || g.pw != 0) return false;
    const int rows = op == CONV2D_FWD ? g.K : g.C, depth = op == CONV2D_FWD ? g.C : g.K;
    if ((int64_t)g.N * depth * g.H * g.W * 4 >= (int64_t(1) << 31)) return false;
    if ((int64_t)g.N * rows * g.H * g.W * 4 >= (int64_t(1) << 31)) return false;
    return pw_stream_lds_bytes(rows, depth) != 0;
}

void fill_pw_args(PwArgs &a, const Geom &g, conv2d_op op, const float *in)
{
    const bool fwd = op == CONV2D_FWD;
    a.in = in;
    a.D = fwd ? g.C : g.K;
    a.Rout = fwd ? g.K : g.C;
    a.HW = g.H * g.W;
    a.M = g.N * a.HW;
    a.ntiles = ceil_div(a.M, 32);
    a.in_bytes = (int32_t)((int64_t)a.M * a.D * 4);
    a.out_bytes = (int32_t)((int64_t)a.M * a.Rout * 4);
    a.w_row_stride = fwd ? g.C : 1;
    a.w_depth_stride = fwd ? 1 : g.C;
    a.depth_fast = fwd ? 1 : 0;
    a.div_HW = make_fastdiv((uint32_t)a.HW);
    a.div_fast = make_fastdiv((uint32_t)(fwd ? a.D : a.Rout));
    a.ngroup = 1;
    for (int i = 0; i <= kMaxGroups; ++i) a.r0[i] = i == 0 ? 0 : a.Rout;
}

// Forward pass of a layer whose filter bank (K x C*R*S) fits in LDS, K <= 128: the taps
// form of the streaming kernel
bool tap_stream_ok(const Geom &g)
{
    if (g.R * g.S == 1 || g.R > 15 || g.S > 15 || g.K > 128) return false;
    if ((int64_t)g.N * g.C * g.H * g.W * 4 >= (int64_t(1) << 31)) return false;
    if ((int64_t)g.N * g.K * g.P * g.Q * 4 >= (int64_t(1) << 31)) return false;
    return pw_stream_lds_bytes(g.K, g.C * g.R * g.S) != 0;
}

void fill_tap_args(PwArgs &a, const Geom &g, const float *x)
{
    a.in = x;
    a.D = g.C * g.R * g.S;
    a.Rout = g.K;
    a.HW = g.P * g.Q;
    a.M = g.N * a.HW;
    a.ntiles = ceil_div(a.M, 32);
    a.in_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    a.out_bytes = (int32_t)((int64_t)a.M * a.Rout * 4);
    a.w_row_stride = a.D;
    a.w_depth_stride = 1;
    a.depth_fast = 1;
    a.div_HW = make_fastdiv((uint32_t)a.HW);
    a.div_fast = make_fastdiv((uint32_t)a.D);
    a.ngroup = 1;
    for (int i = 0; i <= kMaxGroups; ++i) a.r0[i] = i == 0 ? 0 : a.Rout;
    a.tC = g.C; a.tH = g.H; a.tW = g.W; a.tR = g.R; a.tS = g.S;
    a.tsh = g.sh; a.tsw = g.sw; a.tph = g.ph; a.tpw = g.pw; a.tQ = g.Q;
    a.div_tQ = make_fastdiv((uint32_t)g.Q);
}

// Stride-1 backward-data of a layer whose filter bank fits in LDS, C <= 128: the same kernel
// over dy.  Worth it only when the C rows fill a good part of the 32-row MFMA tiles.
bool tap_stream_bwd_ok(const Geom &g)
{
    if (g.sh != 1 || g.sw != 1 || g.R * g.S == 1 || g.R > 15 || g.S > 15 || g.C > 128) return false;
    if ((int64_t)g.N * g.C * g.H * g.W * 4 >= (int64_t(1) << 31)) return false;
    if ((int64_t)g.N * g.K * g.P * g.Q * 4 >= (int64_t(1) << 31)) return false;
    return pw_stream_lds_bytes(g.C, g.K * g.R * g.S) != 0;
}

void fill_tap_bwd_args(PwArgs &a, const Geom &g, const float *dy)
{
    a.in = dy;
    a.D = g.K * g.R * g.S;
    a.Rout = g.C;
    a.HW = g.H * g.W;
    a.M = g.N * a.HW;
    a.ntiles = ceil_div(a.M, 32);
    a.in_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
    a.out_bytes = (int32_t)((int64_t)a.M * a.Rout * 4);
    a.w_row_stride = 0;
    a.w_depth_stride = 0;
    a.depth_fast = 0;
    a.div_HW = make_fastdiv((uint32_t)a.HW);
    a.div_fast = make_fastdiv(1u);
    a.ngroup = 1;
    for (int i = 0; i <= kMaxGroups; ++i) a.r0[i] = i == 0 ? 0 : a.Rout;
    a.tC = g.K; a.tH = g.P; a.tW = g.Q; a.tR = g.R; a.tS = g.S;
    a.tsh = 1; a.tsw = 1; a.tph = g.R - 1 - g.ph; a.tpw = g.S - 1 - g.pw; a.tQ = g.W;
    a.tap_bwd = 1;
    a.div_tQ = make_fastdiv((uint32_t)g.W);
    a.div_tRS = make_fastdiv((uint32_t)(g.R * g.S));
    a.div_rows = make_fastdiv((uint32_t)g.C);
}

// Pointwise backward-weight as a streaming product (pointwise.hip): plan of the split
// of the pixel axis.  ok = the layer qualifies (pointer alignment is checked at the call).
struct PwWgradPlan {
    bool ok;
    int splits, steps_per_split, quads, phases, tiles_c;
    size_t part_bytes, bias_bytes, total_bytes;
};

PwWgradPlan plan_pw_wgrad(const Geom &g)
{
    PwWgradPlan p = {};
    const int HW = g.H * g.W;
    if (g.R != 1 || g.S != 1 || g.sh != 1 || g.sw != 1 || g.ph != 0 || g.pw != 0) return p;
    if (HW % 4 != 0 || HW < 16 || g.K > 128 || g.C > 256) return p;
    if ((int64_t)g.N * g.C * HW * 4 >= (int64_t(1) << 31) || (int64_t)g.N * g.K * HW * 4 >= (int64_t(1) << 31))
        return p;
    p.ok = true;
    p.quads = g.N * (HW / 4);
    const int total_steps = (p.quads + 3) / 4;          // 16 pixels per step
    // one workgroup of column groups x pixel phases waves per split: about eight waves
    // per compute unit, at least four steps per wave; every split costs a K x C partial
    // product to write and add
    int NJ, BT;
    pw_wgrad_shape(g.C, g.K, HW, &NJ, &BT, &p.phases);
    p.tiles_c = NJ;
    int per_cu = 8 / (NJ * p.phases);
    if (per_cu < 1) per_cu = 1;
    int splits = 256 * per_cu;
    if (splits > total_steps / (4 * p.phases)) splits = total_steps / (4 * p.phases);
    if (splits < 1) splits = 1;
    p.steps_per_split = ceil_div(total_steps, splits);
    p.splits = ceil_div(total_steps, p.steps_per_split);
    p.part_bytes = align_up((size_t)p.splits * g.K * g.C * sizeof(float), 256);
    p.bias_bytes = align_up((size_t)p.splits * g.K * sizeof(float), 256);
    p.total_bytes = p.part_bytes + p.bias_bytes;
    return p;
}

// Backward-weight of a small stride-1 filter over very few channels (C*R*S <= 32 taps:
// first layers) with the taps form of the pointwise kernel; same split plan.
PwWgradPlan plan_tap_wgrad(const Geom &g)
{
    PwWgradPlan p = {};
    const int taps = g.C * g.R * g.S, PQ = g.P * g.Q;
    if (g.sh != 1 || g.sw != 1 || g.R * g.S == 1 || taps > 32 || g.K > 128) return p;
    if (g.Q % 4 != 0 || PQ < 16) return p;
    if ((int64_t)g.N * g.C * g.H * g.W * 4 >= (int64_t(1) << 31) || (int64_t)g.N * g.K * PQ * 4 >= (int64_t(1) << 31))
        return p;
    p.ok = true;
    p.quads = g.N * (PQ / 4);
    const int total_steps = (p.quads + 3) / 4;
    int NJ, BT;
    pw_wgrad_shape(taps, g.K, PQ, &NJ, &BT, &p.phases);
    p.tiles_c = NJ;
    int per_cu = 8 / (NJ * p.phases);
    if (per_cu < 1) per_cu = 1;
    int splits = 256 * per_cu;
    if (splits > total_steps / (4 * p.phases)) splits = total_steps / (4 * p.phases);
    if (splits < 1) splits = 1;
    p.steps_per_split = ceil_div(total_steps, splits);
    p.splits = ceil_div(total_steps, p.steps_per_split);
    p.part_bytes = align_up((size_t)p.splits * g.K * taps * sizeof(float), 256);
    p.bias_bytes = align_up((size_t)p.splits * g.K * sizeof(float), 256);
    p.total_bytes = p.part_bytes + p.bias_bytes;
    return p;
}

// first-layer backward-data on the vector ALU: 3x3, stride 1, pad_w 1, C <= 4, rows of
// 4-pixel groups with aligned 16-byte accesses
bool smallc_bwd_ok(const Geom &g, const float *dy, const float *dx)
{
    return g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && g.pw == 1 && g.ph <= 2 && g.C <= 4 &&
           g.W % 4 == 0 && ((uintptr_t)dy & 15) == 0 && ((uintptr_t)dx & 15) == 0 &&
           (int64_t)g.N * g.K * g.P * g.Q * 4 < (int64_t(1) << 31);
}


int run_wino(const Geom &g, conv2d_op op, const float *in, const float *w, const float *bias,
             float *out, void *ws, size_t ws_bytes, hipStream_t s, int relu = 0, int pool = 0)
{
    const WinoPlan p = plan_wino(g, op);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    float *U = (float *)ws;
    int rc = launch_status(launch_wino_filter(w, U, g.K, g.C, g.R, g.S, p.Cin, p.Kout, p.Cpad, p.Kpad,
                                              op == CONV2D_FWD ? 0 : 1, p.mode != 0, s));
    if (rc) return rc;
    WinoArgs a = {};
    a.in = in; a.U = U; a.bias = bias; a.out = out; a.relu = relu; a.pool = pool;
    a.N = g.N; a.Cin = p.Cin; a.Cpad = p.Cpad; a.Hin = p.Hin; a.Win = p.Win;
    a.Kout = p.Kout; a.Kpad = p.Kpad; a.Hout = p.Hout; a.Wout = p.Wout;
    a.pad_h = p.pad_h; a.pad_w = p.pad_w; a.TH = p.TH; a.TW = p.TW; a.T = p.T; a.mode = p.mode;
    a.tiles_t = p.tiles_t; a.tiles_k = p.tiles_k;
    a.nchunks = p.Cpad / wino_chan_chunk();
    a.nsub = p.nsub;
    {
        const int nsw = ceil_div(g.S, 3);
        for (int q = 0; q < 4; ++q) {
            a.sub_dh[q] = q < p.nsub ? 3 * (q / nsw) : 0;
            a.sub_dw[q] = q < p.nsub ? 3 * (q % nsw) : 0;
        }
    }
    a.units_total = p.tiles_t * p.tiles_k * a.nchunks;
    a.partial = (float *)((char *)ws + p.u_bytes);
    a.in_bytes = (int32_t)((int64_t)g.N * p.Cin * p.Hin * p.Win * 4);
    a.u_bytes = (int32_t)((int64_t)16 * p.Cpad * p.Kpad * 4);
    a.vec2 = (p.Wout % 2 == 0) && (((uintptr_t)out & 7) == 0);
    return launch_status(launch_wino_fused(a, p.grid, s));
}

// Winograd backward-weight of a stride-1 layer; acc_w / acc_b: add to dw / dbias
int run_wino_wgrad(const Geom &g, const float *x, const float *dy, float *dw, float *dbias, float scale,
                   int acc_w, int acc_b, void *ws, size_t ws_bytes, hipStream_t s)
{
    const WinoWgradPlan p = plan_wino_wgrad(g);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    float *part = (float *)ws;
    float *bias_part = (float *)((char *)ws + p.part_bytes);
    WinoWgradArgs a = {};
    a.x = x; a.dy = dy; a.part = part; a.bias_part = dbias ? bias_part : nullptr;
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.P = g.P; a.Q = g.Q;
    a.pad_h = g.ph; a.pad_w = g.pw;
    a.TH = p.TH; a.TW = p.TW; a.T = p.T; a.mode = p.mode;
    a.tiles_per_split = p.tiles_per_split;
    a.tiles_k = p.tiles_k; a.tiles_c = p.tiles_c; a.splits = p.splits;
    a.x_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    a.dy_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
    a.div_THW = make_fastdiv((uint32_t)(p.TH * p.TW));
    a.div_TW = make_fastdiv((uint32_t)p.TW);
    a.nsub = p.nsub; a.tiles_c_sub = p.tiles_c_sub;
    {
        const int nsw = ceil_div(g.S, 3);
        for (int q = 0; q < 4; ++q) {
            a.sub_dh[q] = q < p.nsub ? 3 * (q / nsw) : 0;
            a.sub_dw[q] = q < p.nsub ? 3 * (q % nsw) : 0;
        }
    }
    int rc = launch_status(launch_wino_wgrad(a, s));
    if (rc) return rc;
    const BiasJob bj = {dbias ? bias_part : nullptr, dbias, g.K, p.splits, acc_b};
    if (p.nsub > 1)
        rc = launch_status(launch_split_reduce_sub(part, dw, g.K, g.C, g.R, g.S, p.splits, scale, acc_w, bj, s));
    else
        rc = launch_status(launch_split_reduce(part, dw, (int64_t)g.K * g.C * 9, p.splits, scale, acc_w, bj, s));
    return rc;
}

// ---- strided layers as stride-1 3x3 layers over s*s*C channels (space_to_depth.hip) ----
struct S2dPlan {
    bool ok;
    int s, Cq;                  // stride; channels of the rearranged input (s*s*C padded)
    Geom g2;                    // the stride-1 3x3 layer
    size_t x2_bytes, w2_bytes, dw2_bytes, inner_bytes, total_bytes;
};

size_t wino_ws_bytes(const Geom &g, conv2d_op op)
{
    return op == CONV2D_BWD_WEIGHT ? plan_wino_wgrad(g).total_bytes : plan_wino(g, op).total_bytes;
}

S2dPlan plan_s2d(const Geom &g, conv2d_op op)
{
    S2dPlan p = {};
    const int st = g.sh;
    if (st < 2 || st > 4 || g.sw != st) return p;
    if (ceil_div(g.R, st) != 3 || ceil_div(g.S, st) != 3) return p;
    if (g.N > 65535) return p;                              // the rearrangement kernels' grid
    // channel granularity of the Winograd kernels: 8 (chunk) / 32 (backward-weight tile)
    p.Cq = round_up(st * st * g.C, op == CONV2D_BWD_WEIGHT ? 32 : 8);
    if (p.Cq > 65535) return p;
    Geom &q = p.g2;
    q.N = g.N; q.C = p.Cq; q.H = g.P + 2; q.W = g.Q + 2; q.K = g.K; q.R = 3; q.S = 3;
    q.sh = 1; q.sw = 1; q.ph = 0; q.pw = 0; q.P = g.P; q.Q = g.Q;
    if ((int64_t)q.N * q.C * q.H * q.W * 4 >= (int64_t(1) << 31)) return p;
    if (!wino_applicable(q, op)) return p;
    p.ok = true;
    p.s = st;
    p.x2_bytes = align_up((size_t)q.N * q.C * q.H * q.W * sizeof(float), 256);
    p.w2_bytes = align_up((size_t)q.K * q.C * 9 * sizeof(float), 256);
    p.dw2_bytes = op == CONV2D_BWD_WEIGHT ? p.w2_bytes : 0;
    p.inner_bytes = wino_ws_bytes(q, op);
    p.total_bytes = p.x2_bytes + p.w2_bytes + p.dw2_bytes + p.inner_bytes;
    return p;
}

bool s2d_applicable(const Geom &g, conv2d_op op) { return plan_s2d(g, op).ok; }

void fill_s2d_args(S2dArgs &a, const Geom &g, const S2dPlan &p)
{
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.s = p.s; a.pad_h = g.ph; a.pad_w = g.pw;
    a.Cq = p.Cq; a.H2 = p.g2.H; a.W2 = p.g2.W;
    a.I2 = ceil_div(g.H + g.ph, p.s) > a.H2 ? ceil_div(g.H + g.ph, p.s) : a.H2;
    a.J2 = ceil_div(g.W + g.pw, p.s) > a.W2 ? ceil_div(g.W + g.pw, p.s) : a.W2;
    a.div_W2 = make_fastdiv((uint32_t)a.W2);
    a.div_J2 = make_fastdiv((uint32_t)a.J2);
}

int run_s2d(const Geom &g, conv2d_op op, const float *in, const float *w, const float *bias, float *out,
            void *ws, size_t ws_bytes, hipStream_t s, int relu = 0)
{
    const S2dPlan p = plan_s2d(g, op);
    if (!p.ok) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    float *x2 = (float *)ws;
    float *w2 = (float *)((char *)ws + p.x2_bytes);
    void *inner = (char *)ws + p.x2_bytes + p.w2_bytes;
    S2dArgs sa = {};
    fill_s2d_args(sa, g, p);
    int rc = launch_status(launch_filter_s2d(w, w2, g.K, g.C, g.R, g.S, p.s, p.Cq, s));
    if (rc) return rc;
    if (op == CONV2D_FWD) {
        sa.x = in; sa.x2 = x2;
        rc = launch_status(launch_space_to_depth(sa, s));
        if (rc) return rc;
        return run_wino(p.g2, CONV2D_FWD, x2, w2, bias, out, inner, p.inner_bytes, s, relu);
    }
    // backward-data: gradient of the rearranged input, then the inverse permutation
    rc = run_wino(p.g2, CONV2D_BWD_DATA, in, w2, nullptr, x2, inner, p.inner_bytes, s);
    if (rc) return rc;
    sa.x2 = x2; sa.dx = out;
    return launch_status(launch_depth_to_space(sa, s));
}

int run_s2d_wgrad(const Geom &g, const float *x, const float *dy, float *dw, float *dbias, float scale,
                  int accumulate, void *ws, size_t ws_bytes, hipStream_t s)
{
    const S2dPlan p = plan_s2d(g, CONV2D_BWD_WEIGHT);
    if (!p.ok) return CONV2D_ERR_ALGO;
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    float *x2 = (float *)ws;
    float *dw2 = (float *)((char *)ws + p.x2_bytes + p.w2_bytes);
    void *inner = (char *)ws + p.x2_bytes + p.w2_bytes + p.dw2_bytes;
    S2dArgs sa = {};
    fill_s2d_args(sa, g, p);
    sa.x = x; sa.x2 = x2;
    int rc = launch_status(launch_space_to_depth(sa, s));
    if (rc) return rc;
    // scaled gradient of the rearranged filter (not accumulated), then back to K x C x R x S
    rc = run_wino_wgrad(p.g2, x2, dy, dw2, dbias, scale, 0, accumulate, inner, p.inner_bytes, s);
    if (rc) return rc;
    return launch_status(launch_filter_d2s(dw2, dw, g.K, g.C, g.R, g.S, p.s, p.Cq, accumulate, s));
}

}  // namespace

extern "C" {

int conv2d_output_dims(const conv2d_desc *d, int32_t *P, int32_t *Q)
{
    Geom g;
    if (!P || !Q) return CONV2D_ERR_NULL;
    const int rc = check_desc(d, &g);
    if (rc) return rc;
    *P = g.P;
    *Q = g.Q;
    return CONV2D_OK;
}

int conv2d_pick_algo(const conv2d_desc *d, conv2d_op op)
{
    Geom g;
    const int rc = check_desc(d, &g);
    if (rc) return rc;
    if (op != CONV2D_FWD && op != CONV2D_BWD_DATA && op != CONV2D_BWD_WEIGHT) return CONV2D_ERR_ALGO;
    return resolve_algo(g, op, CONV2D_ALGO_AUTO);
}

size_t conv2d_workspace_bytes(const conv2d_desc *d, conv2d_op op, conv2d_algo algo)
{
    Geom g;
    if (check_desc(d, &g)) return 0;
    const int al = resolve_algo(g, op, (int)algo);
    if (al < 0) return 0;
    if (al == CONV2D_ALGO_WINOGRAD)
        return wino_applicable(g, op) ? wino_ws_bytes(g, op) : plan_s2d(g, op).total_bytes;
    if (al == CONV2D_ALGO_WINOGRAD4)
        return op == CONV2D_BWD_WEIGHT ? plan_wino4_wgrad(g).total_bytes : plan_wino4(g, op).total_bytes;
    if (al == CONV2D_ALGO_FFT) return plan_fft(g, op).total_bytes;
    switch (op) {
    case CONV2D_FWD: return plan_fwd(g).total_bytes;
    case CONV2D_BWD_DATA: return plan_bwd_data(g).total_bytes;
    case CONV2D_BWD_WEIGHT: {
        // the streaming pointwise kernel is taken when the pointers allow it: room for either
        size_t bytes = plan_wgrad(g).total_bytes;
        const PwWgradPlan pw = plan_pw_wgrad(g), tw = plan_tap_wgrad(g);
        if (pw.ok && pw.total_bytes > bytes) bytes = pw.total_bytes;
        if (tw.ok && tw.total_bytes > bytes) bytes = tw.total_bytes;
        return bytes;
    }
    default: return 0;
    }
}

static int fwd_impl(const conv2d_desc *d, const float *x, const float *w, const float *bias, float *y,
                    void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream, int relu)
{
    Geom g;
    int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!x || !w || !y) return CONV2D_ERR_NULL;
    const int al = resolve_algo(g, CONV2D_FWD, (int)algo);
    if (al < 0) return al;
    hipStream_t s = (hipStream_t)hip_stream;
    if (al == CONV2D_ALGO_WINOGRAD4) return run_wino4(g, CONV2D_FWD, x, w, bias, y, ws, ws_bytes, s, relu);
    if (al == CONV2D_ALGO_FFT) return run_fft(g, CONV2D_FWD, x, w, bias, y, ws, ws_bytes, s, relu);
    if (al == CONV2D_ALGO_WINOGRAD)
        return wino_applicable(g, CONV2D_FWD) ? run_wino(g, CONV2D_FWD, x, w, bias, y, ws, ws_bytes, s, relu)
                                              : run_s2d(g, CONV2D_FWD, x, w, bias, y, ws, ws_bytes, s, relu);

    const GatherPlan p = plan_fwd(g);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    if (pw_stream_ok(g, CONV2D_FWD)) {
        PwArgs pa = {};
        fill_pw_args(pa, g, CONV2D_FWD, x);
        pa.w[0] = w; pa.bias[0] = bias; pa.out[0] = y; pa.relu = relu;
        pa.fill_vec = g.C % 4 == 0 && ((uintptr_t)w & 15) == 0;
        return launch_status(launch_pw_stream(pa, s));
    }
    if (tap_stream_ok(g)) {
        PwArgs pa = {};
        fill_tap_args(pa, g, x);
        pa.w[0] = w; pa.bias[0] = bias; pa.out[0] = y; pa.relu = relu;
        pa.fill_vec = pa.D % 4 == 0 && ((uintptr_t)w & 15) == 0;
        return launch_status(launch_tap_stream(pa, s));
    }
    float *wt = (float *)ws;
    DepthEntry *tab = (DepthEntry *)((char *)ws + p.wt_bytes);

    PrepArgs pa = {};
    pa.w = w; pa.wt = wt; pa.tab = tab; pa.mode = 0;
    pa.K = g.K; pa.C = g.C; pa.R = g.R; pa.S = g.S; pa.Kpad = p.Kpad;
    pa.gather_chan_stride = g.H * g.W; pa.gather_W = g.W;
    pa.stride_h = g.sh; pa.stride_w = g.sw;
    pa.rows_total = (int32_t)p.rows_total; pa.nphases = 1;
    pa.ph[0].row0 = 0; pa.ph[0].rows = g.C * g.R * g.S; pa.ph[0].rows_pad = (int32_t)p.rows_total;
    rc = launch_status(launch_gemmconv_prep(pa, s));
    if (rc) return rc;

    GemmConvArgs a = {};
    a.in = x; a.wt = wt; a.tab = tab; a.bias = bias; a.out = y; a.relu = relu;
    a.N = g.N; a.Hin = g.H; a.Win = g.W; a.in_img_stride = g.C * g.H * g.W;
    a.Kout = g.K; a.Kpad = p.Kpad; a.Hout = g.P; a.Wout = g.Q;
    a.out_chan_stride = g.P * g.Q; a.out_img_stride = g.K * g.P * g.Q;
    a.in_step_h = g.sh; a.in_step_w = g.sw; a.out_step_h = 1; a.out_step_w = 1;
    a.tiles_k = p.Kpad / gemmconv_filter_tile(p.tile);
    a.tiles_pix = ceil_div(g.N * g.P * g.Q, gemmconv_pixel_tile(p.tile));
    a.phase[0].row0 = 0;
    a.phase[0].depth_tiles = (int32_t)(p.rows_total / kDepthTile);
    a.phase[0].in_base_h = -g.ph; a.phase[0].in_base_w = -g.pw;
    a.phase[0].out_base_h = 0; a.phase[0].out_base_w = 0;
    a.phase[0].Hs = g.P; a.phase[0].Ws = g.Q;
    if (pointwise_ok(g, x, (int64_t)g.N * g.C * g.H * g.W)) {
        a.pw_depth = g.C;
        a.in_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    }
    return run_gemmconv(a, p.tile, 1, g, 1.0, s);
}

int conv2d_fwd(const conv2d_desc *d, const float *x, const float *w, const float *bias, float *y,
               void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream)
{
    return fwd_impl(d, x, w, bias, y, ws, ws_bytes, algo, hip_stream, 0);
}

int conv2d_fwd_relu(const conv2d_desc *d, const float *x, const float *w, const float *bias, float *y,
                    void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream)
{
    return fwd_impl(d, x, w, bias, y, ws, ws_bytes, algo, hip_stream, 1);
}

int conv2d_fwd_static(const conv2d_desc *d, const float *x, const float *w, const float *bias, float *y,
                      conv2d_algo algo, void *hip_stream)
{
    Geom g;
    int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!x || !w || !y) return CONV2D_ERR_NULL;
    const int al = resolve_algo(g, CONV2D_FWD, (int)algo);
    if (al < 0) return al;
    // what conv2d_fwd would ask of the caller; nothing in it has to start at zero (the
    // filter matrix / transformed filters and the cut-tile slots are written before they
    // are read), so the last call's contents may stay
    size_t need = conv2d_workspace_bytes(d, CONV2D_FWD, algo);
    if (need == 0) return CONV2D_ERR_ALGO;
    // AUTO may pick the unfused Winograd path, whose workspace holds whole transformed
    // tensors: where that does not fit, take the fused kernels, which need far less
    if (need > (size_t)CONV2D_STATIC_SCRATCH_BYTES && algo == CONV2D_ALGO_AUTO && (al == CONV2D_ALGO_WINOGRAD4 || al == CONV2D_ALGO_FFT)) {
        algo = CONV2D_ALGO_WINOGRAD;
        need = conv2d_workspace_bytes(d, CONV2D_FWD, algo);
        if (need == 0) return CONV2D_ERR_ALGO;
    }
    if (need > (size_t)CONV2D_STATIC_SCRATCH_BYTES) return CONV2D_ERR_STATIC_LIMIT;
    void *ws = static_scratch(&rc);
    if (!ws) return rc;
    return fwd_impl(d, x, w, bias, y, ws, (size_t)CONV2D_STATIC_SCRATCH_BYTES, algo, hip_stream, 0);
}

int conv2d_fwd_relu_pool2(const conv2d_desc *d, const float *x, const float *w, const float *bias,
                          float *y_pooled, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    const int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!x || !w || !y_pooled) return CONV2D_ERR_NULL;
    // the Winograd kernels' 2x2 output blocks are the pooling windows
    if (!wino_applicable(g, CONV2D_FWD) || g.P % 2 != 0 || g.Q % 2 != 0) return CONV2D_ERR_ALGO;
    return run_wino(g, CONV2D_FWD, x, w, bias, y_pooled, ws, ws_bytes, (hipStream_t)hip_stream, 1, 1);
}

int conv2d_fwd_1x1_group(const conv2d_desc *d, const float *x, int32_t ngroup, const int32_t *K,
                         const float *const *w, const float *const *bias, float *const *y, void *ws,
                         size_t ws_bytes, void *hip_stream)
{
    Geom g;
    int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!x || !K || !w || !y) return CONV2D_ERR_NULL;
    if (ngroup < 1 || ngroup > kMaxGroups) return CONV2D_ERR_GEOMETRY;
    if (g.R != 1 || g.S != 1 || g.sh != 1 || g.sw != 1 || g.ph != 0 || g.pw != 0) return CONV2D_ERR_ALGO;
    int ksum = 0;
    for (int i = 0; i < ngroup; ++i) {
        if (K[i] < 1) return CONV2D_ERR_GEOMETRY;
        if (!w[i] || !y[i]) return CONV2D_ERR_NULL;
        ksum += K[i];
    }
    if (ksum != g.K) return CONV2D_ERR_GEOMETRY;
    hipStream_t s = (hipStream_t)hip_stream;

    const GatherPlan p = plan_fwd(g);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    if (pw_stream_ok(g, CONV2D_FWD)) {
        PwArgs sa = {};
        fill_pw_args(sa, g, CONV2D_FWD, x);
        sa.ngroup = ngroup;
        int r = 0;
        for (int i = 0; i < kMaxGroups; ++i) {
            const bool used = i < ngroup;
            sa.r0[i] = r;
            sa.w[i] = used ? w[i] : w[0];
            sa.bias[i] = (used && bias) ? bias[i] : nullptr;
            sa.out[i] = used ? y[i] : y[0];
            if (used) r += K[i];
        }
        sa.r0[kMaxGroups] = r;
        sa.fill_vec = g.C % 4 == 0;
        for (int i = 0; i < ngroup; ++i)
            if (((uintptr_t)w[i] & 15) != 0) sa.fill_vec = 0;
        return launch_status(launch_pw_stream(sa, s));
    }
    float *wt = (float *)ws;
    DepthEntry *tab = (DepthEntry *)((char *)ws + p.wt_bytes);

    PrepArgs pa = {};
    pa.w = nullptr; pa.wt = wt; pa.tab = tab; pa.mode = 3;
    pa.K = g.K; pa.C = g.C; pa.R = 1; pa.S = 1; pa.Kpad = p.Kpad;
    pa.gather_chan_stride = g.H * g.W; pa.gather_W = g.W;
    pa.stride_h = 1; pa.stride_w = 1;
    pa.rows_total = (int32_t)p.rows_total; pa.nphases = 1;
    pa.ph[0].row0 = 0; pa.ph[0].rows = g.C; pa.ph[0].rows_pad = (int32_t)p.rows_total;

    GemmConvArgs a = {};
    a.in = x; a.wt = wt; a.tab = tab; a.bias = nullptr; a.out = y[0];
    a.N = g.N; a.Hin = g.H; a.Win = g.W; a.in_img_stride = g.C * g.H * g.W;
    a.Kout = g.K; a.Kpad = p.Kpad; a.Hout = g.P; a.Wout = g.Q;
    a.out_chan_stride = g.P * g.Q; a.out_img_stride = g.K * g.P * g.Q;
    a.in_step_h = 1; a.in_step_w = 1; a.out_step_h = 1; a.out_step_w = 1;
    a.tiles_k = p.Kpad / gemmconv_filter_tile(p.tile);
    a.tiles_pix = ceil_div(g.N * g.P * g.Q, gemmconv_pixel_tile(p.tile));
    a.phase[0].row0 = 0;
    a.phase[0].depth_tiles = (int32_t)(p.rows_total / kDepthTile);
    a.phase[0].in_base_h = 0; a.phase[0].in_base_w = 0;
    a.phase[0].out_base_h = 0; a.phase[0].out_base_w = 0;
    a.phase[0].Hs = g.P; a.phase[0].Ws = g.Q;
    a.ngroup = ngroup;
    int k0 = 0;
    for (int i = 0; i <= kMaxGroups; ++i) {
        pa.gk0[i] = k0;
        a.grp_k0[i] = k0;
        if (i < kMaxGroups) {
            const bool used = i < ngroup;
            pa.gw[i] = used ? w[i] : w[0];
            a.grp_out[i] = used ? y[i] : y[0];
            a.grp_bias[i] = (used && bias) ? bias[i] : nullptr;
            if (used) k0 += K[i];
        }
    }
    rc = launch_status(launch_gemmconv_prep(pa, s));
    if (rc) return rc;
    if (pointwise_ok(g, x, (int64_t)g.N * g.C * g.H * g.W)) {
        a.pw_depth = g.C;
        a.in_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
    }
    return run_gemmconv(a, p.tile, 1, g, 1.0, s);
}

int conv2d_bwd_data(const conv2d_desc *d, const float *dy, const float *w, float *dx, void *ws,
                    size_t ws_bytes, conv2d_algo algo, void *hip_stream)
{
    Geom g;
    int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!dy || !w || !dx) return CONV2D_ERR_NULL;
    const int al = resolve_algo(g, CONV2D_BWD_DATA, (int)algo);
    if (al < 0) return al;
    hipStream_t s = (hipStream_t)hip_stream;
    if (algo == CONV2D_ALGO_AUTO && smallc_bwd_ok(g, dy, dx)) {
        SmallCArgs sa = {};
        sa.dy = dy; sa.w = w; sa.dx = dx;
        sa.N = g.N; sa.C = g.C; sa.H = g.H; sa.W = g.W; sa.K = g.K; sa.P = g.P; sa.Q = g.Q; sa.pad_h = g.ph;
        sa.dy_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
        return launch_status(launch_bwd_data_smallc(sa, s));
    }
    if (al == CONV2D_ALGO_WINOGRAD4) return run_wino4(g, CONV2D_BWD_DATA, dy, w, nullptr, dx, ws, ws_bytes, s);
    if (al == CONV2D_ALGO_FFT) return run_fft(g, CONV2D_BWD_DATA, dy, w, nullptr, dx, ws, ws_bytes, s);
    if (al == CONV2D_ALGO_WINOGRAD)
        return wino_applicable(g, CONV2D_BWD_DATA)
                   ? run_wino(g, CONV2D_BWD_DATA, dy, w, nullptr, dx, ws, ws_bytes, s)
                   : run_s2d(g, CONV2D_BWD_DATA, dy, w, nullptr, dx, ws, ws_bytes, s);

    const GatherPlan p = plan_bwd_data(g);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    if (pw_stream_ok(g, CONV2D_BWD_DATA)) {
        PwArgs pa = {};
        fill_pw_args(pa, g, CONV2D_BWD_DATA, dy);
        pa.w[0] = w; pa.bias[0] = nullptr; pa.out[0] = dx;
        pa.fill_vec = g.C % 4 == 0 && ((uintptr_t)w & 15) == 0;
        return launch_status(launch_pw_stream(pa, s));
    }
    if (tap_stream_bwd_ok(g) && g.C >= kTapBwdMinRows) {
        PwArgs pa = {};
        fill_tap_bwd_args(pa, g, dy);
        pa.w[0] = w; pa.bias[0] = nullptr; pa.out[0] = dx;
        return launch_status(launch_tap_stream(pa, s));
    }
    float *wt = (float *)ws;
    DepthEntry *tab = (DepthEntry *)((char *)ws + p.wt_bytes);
    const int BN = gemmconv_pixel_tile(p.tile);

    GemmConvArgs a = {};
    a.in = dy; a.wt = wt; a.tab = tab; a.bias = nullptr; a.out = dx;
    a.N = g.N; a.Hin = g.P; a.Win = g.Q; a.in_img_stride = g.K * g.P * g.Q;
    a.Kout = g.C; a.Kpad = p.Kpad; a.Hout = g.H; a.Wout = g.W;
    a.out_chan_stride = g.H * g.W; a.out_img_stride = g.C * g.H * g.W;
    a.in_step_h = 1; a.in_step_w = 1; a.out_step_h = g.sh; a.out_step_w = g.sw;
    a.tiles_k = p.Kpad / gemmconv_filter_tile(p.tile);

    if (p.d2s) {
        PrepArgs pa = {};
        pa.w = w; pa.wt = wt; pa.tab = tab; pa.mode = 2;
        pa.K = g.K; pa.C = g.C; pa.R = g.R; pa.S = g.S; pa.Kpad = p.Kpad;
        pa.gather_chan_stride = g.P * g.Q; pa.gather_W = g.Q;
        pa.stride_h = g.sh; pa.stride_w = g.sw; pa.pad_h = g.ph; pa.pad_w = g.pw;
        pa.dr_min = p.dr_min; pa.nd_r = p.nd_r; pa.dt_min = p.dt_min; pa.nd_t = p.nd_t;
        pa.nphases = 1;
        pa.rows_total = (int32_t)p.rows_total;
        pa.ph[0].row0 = 0; pa.ph[0].rows = g.K * p.nd_r * p.nd_t; pa.ph[0].rows_pad = (int32_t)p.rows_total;
        rc = launch_status(launch_gemmconv_prep(pa, s));
        if (rc) return rc;
        const int Hs = ceil_div(g.H, g.sh), Ws = ceil_div(g.W, g.sw);
        a.Kout = g.sh * g.sw * g.C;
        a.d2s_C = g.C; a.d2s_sh = g.sh; a.d2s_sw = g.sw;
        a.div_d2s_C = make_fastdiv((uint32_t)g.C);
        a.div_d2s_sw = make_fastdiv((uint32_t)g.sw);
        a.tiles_pix = ceil_div(g.N * Hs * Ws, BN);
        a.phase[0].row0 = 0;
        a.phase[0].depth_tiles = (int32_t)(p.rows_total / kDepthTile);
        a.phase[0].in_base_h = 0; a.phase[0].in_base_w = 0;
        a.phase[0].out_base_h = 0; a.phase[0].out_base_w = 0;
        a.phase[0].Hs = Hs; a.phase[0].Ws = Ws;
        return run_gemmconv(a, p.tile, 1, g, 1.0, s);
    }

    // phases are prepared and launched in groups of at most kMaxPhases
    int64_t row_cursor = 0;
    for (int first = 0; first < p.nphases; first += kMaxPhases) {
        const int cnt = (p.nphases - first) < kMaxPhases ? (p.nphases - first) : kMaxPhases;
        PrepArgs pa = {};
        pa.w = w; pa.wt = wt + row_cursor * p.Kpad; pa.tab = tab + row_cursor; pa.mode = 1;
        pa.K = g.K; pa.C = g.C; pa.R = g.R; pa.S = g.S; pa.Kpad = p.Kpad;
        pa.gather_chan_stride = g.P * g.Q; pa.gather_W = g.Q;
        pa.stride_h = g.sh; pa.stride_w = g.sw;
        pa.nphases = cnt;
        int32_t group_rows = 0;
        int tiles_pix = 1;
        for (int i = 0; i < cnt; ++i) {
            const int id = first + i;
            const PhaseGeom pg = bwd_phase(g, id / g.sw, id % g.sw);
            pa.ph[i].row0 = group_rows; pa.ph[i].rows = pg.rows; pa.ph[i].rows_pad = pg.rows_pad;
            pa.ph[i].r0 = pg.r0; pa.ph[i].nr = pg.nr; pa.ph[i].t0 = pg.t0; pa.ph[i].nt = pg.nt;
            a.phase[i].row0 = (int32_t)(row_cursor + group_rows);
            a.phase[i].depth_tiles = pg.rows_pad / kDepthTile;
            a.phase[i].in_base_h = pg.in_base_h; a.phase[i].in_base_w = pg.in_base_w;
            a.phase[i].out_base_h = pg.a; a.phase[i].out_base_w = pg.b;
            a.phase[i].Hs = pg.Hs; a.phase[i].Ws = pg.Ws;
            const int tp = ceil_div(g.N * pg.Hs * pg.Ws, BN);
            if (tp > tiles_pix) tiles_pix = tp;
            group_rows += pg.rows_pad;
        }
        pa.rows_total = group_rows;
        if (group_rows > 0) {
            rc = launch_status(launch_gemmconv_prep(pa, s));
            if (rc) return rc;
        }
        a.tiles_pix = tiles_pix;
        if (pointwise_ok(g, dy, (int64_t)g.N * g.K * g.P * g.Q)) {     // implies a single phase
            a.pw_depth = g.K;
            a.in_bytes = (int32_t)((int64_t)g.N * g.K * g.P * g.Q * 4);
        }
        rc = run_gemmconv(a, p.tile, cnt, g, (double)cnt / p.nphases, s);
        if (rc) return rc;
        row_cursor += group_rows;
    }
    return CONV2D_OK;
}

int conv2d_bwd_weight(const conv2d_desc *d, const float *x, const float *dy, float *dw,
                      float *dbias, float scale, int accumulate, void *ws, size_t ws_bytes,
                      conv2d_algo algo, void *hip_stream)
{
    Geom g;
    int rc = check_desc(d, &g);
    if (rc) return rc;
    if (!x || !dy || !dw) return CONV2D_ERR_NULL;
    const int al = resolve_algo(g, CONV2D_BWD_WEIGHT, (int)algo);
    if (al < 0) return al;
    hipStream_t s = (hipStream_t)hip_stream;

    if (al == CONV2D_ALGO_WINOGRAD4) return run_wino4_wgrad(g, x, dy, dw, dbias, scale, accumulate, ws, ws_bytes, s);
    if (al == CONV2D_ALGO_FFT) return run_fft_wgrad(g, x, dy, dw, dbias, scale, accumulate, ws, ws_bytes, s);
    if (al == CONV2D_ALGO_WINOGRAD) {
        if (!wino_applicable(g, CONV2D_BWD_WEIGHT))
            return run_s2d_wgrad(g, x, dy, dw, dbias, scale, accumulate, ws, ws_bytes, s);
        return run_wino_wgrad(g, x, dy, dw, dbias, scale, accumulate, accumulate, ws, ws_bytes, s);
    }

    const PwWgradPlan pw = plan_pw_wgrad(g);
    if (pw.ok && (((uintptr_t)x | (uintptr_t)dy) & 15) == 0) {
        if (!ws_ok(ws, ws_bytes, pw.total_bytes)) return CONV2D_ERR_WORKSPACE;
        float *part = (float *)ws;
        float *bias_part = (float *)((char *)ws + pw.part_bytes);
        PwWgradArgs a = {};
        a.x = x; a.dy = dy; a.part = part; a.bias_part = dbias ? bias_part : nullptr;
        a.N = g.N; a.C = g.C; a.K = g.K; a.HW = g.H * g.W;
        a.x_bytes = (int32_t)((int64_t)g.N * g.C * a.HW * 4);
        a.dy_bytes = (int32_t)((int64_t)g.N * g.K * a.HW * 4);
        a.quads = pw.quads; a.steps_per_split = pw.steps_per_split; a.splits = pw.splits;
        a.tiles_c = pw.tiles_c; a.phases = pw.phases;
        a.div_QW = make_fastdiv((uint32_t)(a.HW / 4));
        rc = launch_status(launch_pw_wgrad(a, s));
        if (rc) return rc;
        const BiasJob bj = {dbias ? bias_part : nullptr, dbias, g.K, pw.splits, accumulate};
        return launch_status(launch_split_reduce(part, dw, (int64_t)g.K * g.C, pw.splits, scale, accumulate, bj, s));
    }

    const PwWgradPlan tw = plan_tap_wgrad(g);
    if (tw.ok && ((uintptr_t)dy & 15) == 0) {
        if (!ws_ok(ws, ws_bytes, tw.total_bytes)) return CONV2D_ERR_WORKSPACE;
        float *part = (float *)ws;
        float *bias_part = (float *)((char *)ws + tw.part_bytes);
        const int taps = g.C * g.R * g.S, PQ = g.P * g.Q;
        PwWgradArgs a = {};
        a.x = x; a.dy = dy; a.part = part; a.bias_part = dbias ? bias_part : nullptr;
        a.N = g.N; a.C = taps; a.K = g.K; a.HW = PQ;
        a.x_bytes = (int32_t)((int64_t)g.N * g.C * g.H * g.W * 4);
        a.dy_bytes = (int32_t)((int64_t)g.N * g.K * PQ * 4);
        a.quads = tw.quads; a.steps_per_split = tw.steps_per_split; a.splits = tw.splits;
        a.tiles_c = tw.tiles_c; a.phases = tw.phases;
        a.div_QW = make_fastdiv((uint32_t)(PQ / 4));
        a.xC = g.C; a.xH = g.H; a.xW = g.W; a.tP = g.P; a.Qd = g.Q; a.tR = g.R; a.tS = g.S; a.tph = g.ph; a.tpw = g.pw;
        a.div_Q = make_fastdiv((uint32_t)g.Q);
        a.div_RS = make_fastdiv((uint32_t)(g.R * g.S));
        a.div_S = make_fastdiv((uint32_t)g.S);
        rc = launch_status(launch_tap_wgrad(a, s));
        if (rc) return rc;
        const BiasJob bj = {dbias ? bias_part : nullptr, dbias, g.K, tw.splits, accumulate};
        return launch_status(launch_split_reduce(part, dw, (int64_t)g.K * taps, tw.splits, scale, accumulate, bj, s));
    }

    const WgradPlan p = plan_wgrad(g);
    if (!ws_ok(ws, ws_bytes, p.total_bytes)) return CONV2D_ERR_WORKSPACE;
    float *part = (float *)ws;
    float *bias_part = (float *)((char *)ws + p.part_bytes);

    WgradArgs a = {};
    a.x = x; a.dy = dy; a.part = part; a.bias_part = dbias ? bias_part : nullptr;
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.R = g.R; a.S = g.S; a.P = g.P; a.Q = g.Q;
    a.stride_h = g.sh; a.stride_w = g.sw; a.pad_h = g.ph; a.pad_w = g.pw;
    a.PQ = g.P * g.Q; a.CRS = g.C * g.R * g.S; a.M = g.N * g.P * g.Q;
    a.chunk = p.chunk; a.tiles_k = p.tiles_k; a.tiles_j = p.tiles_j; a.splits = p.splits;
    a.div_PQ = make_fastdiv((uint32_t)a.PQ);
    a.div_Q = make_fastdiv((uint32_t)g.Q);
    a.div_RS = make_fastdiv((uint32_t)(g.R * g.S));
    a.div_S = make_fastdiv((uint32_t)g.S);
    rc = launch_status(launch_wgrad(a, p.tile, s));
    if (rc) return rc;
    const BiasJob bj = {dbias ? bias_part : nullptr, dbias, g.K, p.splits, accumulate};
    rc = launch_status(launch_split_reduce(part, dw, (int64_t)g.K * a.CRS, p.splits, scale, accumulate, bj, s));
    if (rc) return rc;
    return CONV2D_OK;
}

int apply_mul_add(const float *x, float *y, int64_t n, float a, float b, void *hip_stream)
{
    if (n < 0) return CONV2D_ERR_GEOMETRY;
    if (n == 0) return CONV2D_OK;
    if (!x || !y) return CONV2D_ERR_NULL;
    return launch_status(launch_apply_mul_add(x, y, n, a, b, (hipStream_t)hip_stream));
}

const char *conv2d_status_string(int status)
{
    switch (status) {
    case CONV2D_OK: return "ok";
    case CONV2D_ERR_NULL: return "null descriptor or pointer";
    case CONV2D_ERR_GEOMETRY: return "invalid convolution geometry";
    case CONV2D_ERR_ALGO: return "algorithm not applicable to this geometry";
    case CONV2D_ERR_WORKSPACE: return "workspace missing or too small";
    case CONV2D_ERR_LAUNCH: return "HIP launch error";
    case CONV2D_ERR_STATIC_LIMIT: return "layer needs more workspace than the library's static scratch area holds";
    default: return "unknown status";
    }
}

const char *conv2d_version(void) { return "mi355conv 0.1 (gfx950)"; }

}  // extern "C"
