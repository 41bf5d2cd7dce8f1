// Internal declarations shared by the HIP translation units of libmi355conv.
// Nothing here is part of the C ABI (see include/mi355conv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mi355conv {

// ---------------------------------------------------------------------------
// Division by a run-time constant for numerators below 2^31 (Granlund &
// Montgomery round-up method): q = (mulhi(n, mul) + n) >> shift.
// ---------------------------------------------------------------------------
struct FastDiv {
    uint32_t d, mul, shift;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;
    f.mul = (uint32_t)(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
    f.shift = l;
    return f;
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv &f)
{
    return (__umulhi(n, f.mul) + n) >> f.shift;
}

// ---------------------------------------------------------------------------
// Implicit GEMM, "gather" form, used by forward and backward-data.
//
//   out[n, ko, h, v] = bias[ko] + sum_d  Wt[d][ko] * in[n, chan(d), ih0+dr(d), iw0+dt(d)]
//
// d runs over the rows of the lowered matrix (Sec. 4.2 "implicitgemm": the
// lowered matrix is only ever formed on chip).  A row is described by a table
// entry: the element offset chan*Hin*Win + dr*Win + dt and the signed tap
// displacement (dr, dt) used for the zero-padding test.  Output pixels are
// enumerated on a sub-grid ("phase"): (oh', ow') -> h = oh'*out_step + out_base,
// ih0 = oh'*in_step + in_base.  Forward has one phase (out_step 1, in_step =
// stride, in_base = -pad).  Backward-data has stride_h*stride_w phases, each a
// stride-1 gather from dy with its own subset of the filter taps.
// ---------------------------------------------------------------------------
constexpr int kDepthTile = 16;   // rows of the lowered matrix per main-loop step
constexpr int kMaxPhases = 16;   // phases per launch

struct DepthEntry {
    int32_t off;    // chan*Hin*Win + dr*Win + dt   (elements)
    int32_t drdt;   // (dr << 16) | (dt & 0xffff), both signed 16-bit
};
constexpr int32_t kInvalidDr = 0x4000;   // a dr no image height reaches

struct Phase {
    int32_t row0;          // first row of this phase in Wt / the table
    int32_t depth_tiles;   // padded rows / kDepthTile
    int32_t in_base_h, in_base_w;
    int32_t out_base_h, out_base_w;
    int32_t Hs, Ws;        // sub-grid size
};

constexpr int kMaxGroups = 4;

struct GemmConvArgs {
    const float *in;
    const float *wt;           // [rows_total][Kpad]
    const DepthEntry *tab;     // [rows_total]
    const float *bias;         // nullable
    int32_t relu;              // forward: y = max(0, product + bias)
    float *out;
    int32_t N, Hin, Win, in_img_stride;
    int32_t Kout, Kpad, Hout, Wout, out_chan_stride, out_img_stride;
    int32_t in_step_h, in_step_w, out_step_h, out_step_w;
    int32_t tiles_k, tiles_pix;   // grid.x = tiles_k * tiles_pix (max over phases)
    // depth-to-space epilogue (strided backward-data with few channels): GEMM row
    // k' = (a*d2s_sw + b)*d2s_C + c is stored to out[n][c][oh*d2s_sh + a][ow*d2s_sw + b];
    // d2s_C == 0 selects the ordinary epilogue
    int32_t d2s_C, d2s_sh, d2s_sw;
    FastDiv div_d2s_C, div_d2s_sw;
    // pointwise fast path (1x1, stride 1, no padding, H*W % 4 == 0): pw_depth = number
    // of channels of `in` (0 selects the gather path), in_bytes = its size (< 2^31)
    int32_t pw_depth, in_bytes;
    // grouped outputs (several convolutions of the same input in one pass): GEMM rows
    // grp_k0[g] .. grp_k0[g+1]-1 are the filters of group g and go to grp_out[g]
    // (N x K_g x Hout x Wout) with grp_bias[g] (nullable); ngroup == 0: single output
    int32_t ngroup;
    int32_t grp_k0[kMaxGroups + 1];
    float *grp_out[kMaxGroups];
    const float *grp_bias[kMaxGroups];
    Phase phase[kMaxPhases];
};

struct PrepPhase {
    int32_t row0, rows, rows_pad;
    int32_t r0, nr, t0, nt;     // backward-data: taps r = r0 + i*stride_h, i < nr
};

struct PrepArgs {
    const float *w;
    float *wt;
    DepthEntry *tab;
    int32_t mode;               // 0 forward, 1 backward-data by phases, 2 backward-data
                                //   as one stride-1 gather with depth-to-space rows,
                                //   3 forward with the filters of several groups stacked
    const float *gw[kMaxGroups];        // mode 3: filters of group g, columns gk0[g] .. gk0[g+1]-1
    int32_t gk0[kMaxGroups + 1];
    int32_t K, C, R, S, Kpad;   // Kpad = row pitch of wt
    int32_t gather_chan_stride, gather_W;   // of the tensor the main kernel gathers from
    int32_t stride_h, stride_w;
    int32_t rows_total, nphases;
    int32_t pad_h, pad_w;       // mode 2
    int32_t dr_min, nd_r, dt_min, nd_t;   // mode 2: tap displacements dr_min .. dr_min+nd_r-1
    PrepPhase ph[kMaxPhases];
};

// gather tile = 0: 128 filters x 128 pixels, 1: 64 x 256, 2: 32 x 256, 3: 96 x 128
int gemmconv_filter_tile(int tile);
int gemmconv_pixel_tile(int tile);
hipError_t launch_gemmconv_prep(const PrepArgs &a, hipStream_t s);
hipError_t launch_gemmconv(const GemmConvArgs &a, int tile, int nphases, hipStream_t s);

// ---------------------------------------------------------------------------
// Backward-weight implicit GEMM:  D[k][j] = sum_m dy[m][k] * lowered(x)[m][j],
// m = (n,p,q) output pixels (the reduction over the batch), j = (c,r,s).
// The reduction range is split over `splits` workgroups per output tile; each
// writes its partial tile to `part` and a second kernel adds them in order.
// ---------------------------------------------------------------------------
struct WgradArgs {
    const float *x;
    const float *dy;
    float *part;               // [splits][K][CRS]
    float *bias_part;          // [splits][K] partial sums of dy per filter, or null
    int32_t N, C, H, W, K, R, S, P, Q;
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t PQ, CRS, M;        // M = N*P*Q
    int32_t chunk;             // pixels per split (multiple of the depth step)
    int32_t tiles_k, tiles_j, splits;
    FastDiv div_PQ, div_Q, div_RS, div_S;
};

int wgrad_filter_tile(int tile);
int wgrad_col_tile(int tile);
hipError_t launch_wgrad(const WgradArgs &a, int tile, hipStream_t s);
// Final stage of the bias gradient, done by extra workgroups of the split-reduce launch:
// db[k] = scale * sum_i part[i][k] (+ db[k]).  part == nullptr: no bias gradient wanted.
struct BiasJob {
    const float *part;         // [nsplit][K]
    float *db;
    int32_t K, nsplit, accumulate;
};
// dst[i] = scale * sum_s part[s][i] (+ dst[i] if accumulate)
hipError_t launch_split_reduce(const float *part, float *dst, int64_t count, int splits,
                               float scale, int accumulate, const BiasJob &bj, hipStream_t s);
// dw[k][c][r][s] = scale * sum over splits of part[split][k][q*C + c][(r%3)*3 + s%3], q the
// sub-filter holding tap (r, s) (see WinoWgradArgs)
hipError_t launch_split_reduce_sub(const float *part, float *dw, int K, int C, int R, int S, int splits,
                                   float scale, int accumulate, const BiasJob &bj, hipStream_t s);
// ---------------------------------------------------------------------------
// Winograd F(2x2,3x3), fused (see winograd.hip).  `in` is the tensor the 4x4
// patches are read from (x for forward, dy for backward-data), U the
// transformed filters [16][Cpad][Kpad].
// ---------------------------------------------------------------------------
struct WinoArgs {
    const float *in;
    const float *U;
    const float *bias;       // nullable
    int32_t relu;            // forward: y = max(0, product + bias)
    int32_t pool;            // with relu, Hout and Wout even: out is the 2x2 / stride-2 max-pooled map
                             // [N][Kout][Hout/2][Wout/2] (one pixel per tile)
    float *out;
    int32_t N, Cin, Cpad, Hin, Win, Kout, Kpad, Hout, Wout;
    int32_t pad_h, pad_w;    // patch origin = 2*tile - pad
    int32_t TH, TW, T;       // tiles per image (rows, cols), tiles in total
    int32_t mode;            // 0 one tile per lane; 1 tile pairs (TW even, pad_w 1, even
                             // width), needs the paired U layout
    int32_t tiles_t, tiles_k;
    int32_t vec2;            // output rows can be stored as aligned float2
    int32_t in_bytes, u_bytes;   // sizes of `in` and `U` (both below 2^31)
    int32_t nchunks, units_total; // 8-channel chunks per tile; tiles_t*tiles_k*nchunks
    // filters larger than 3x3 as a sum of 3x3 sub-filters of shifted inputs: the
    // reduction runs over nsub groups of Cin channels (nchunks = nsub * Cin / 8); group q
    // reads the input shifted by (sub_dh[q], sub_dw[q]).  nsub = 1, shifts 0: plain 3x3
    int32_t nsub, sub_dh[4], sub_dw[4];
    float *partial;              // [grid][2] slots of 64*64*4 floats for tiles cut by a range boundary
};

int wino_filter_tile();
int wino_tile_block();
int wino_chan_chunk();
// R x S: the full filter; its 3x3 sub-filter (a, b) holds taps (3a.., 3b..), zero where
// the filter ends; Cpad = nsub * Cin virtual channels, group q = a * ceil(S/3) + b
hipError_t launch_wino_filter(const float *w, float *U, int K, int C, int R, int S, int Cin, int Kout,
                              int Cpad, int Kpad, int mode, int paired, hipStream_t s);
int wino_partial_slot_floats();
// G persistent workgroups (G <= tiles_t*tiles_k)
hipError_t launch_wino_fused(const WinoArgs &a, int G, hipStream_t s);

// Winograd F(4x4,3x3) with separate transform kernels around 36 batched GEMMs (see
// wino4.hip).  `in` is x (forward) or dy (backward-data, with the rotated filter: mode 1).
struct W4Args {
    const float *in;
    const float *w;            // [K][C][3][3]
    const float *bias;         // nullable
    float *out;
    float *U, *V, *M;          // workspace: transformed filters, input tiles, products
    float *slots;              // workspace: [split_tiles][split] partial GEMM tiles
    int32_t split, split_tiles; // the last split_tiles GEMM tiles are computed as `split` depth shares each
                                // (split <= 1: every tile by one workgroup)
    int32_t relu;
    int32_t mode;              // filter transform: 0 forward, 1 backward-data
    int32_t C;                 // channel count of w (its second axis)
    int32_t N, Cin, Hin, Win, Kout, Kpad, Hout, Wout, pad_h, pad_w;
    int32_t TH, TW, T, Tpad;   // 4x4 output tiles per image (rows, cols), in total, padded to the GEMM tile
    int32_t chunks;            // 8-channel chunks of the reduction: nsub * csub
    int32_t R, S;              // filter size (3..6); nsub = ceil(R/3)*ceil(S/3) sub-filters of 3x3
    int32_t csub, nsw;         // chunks per sub-filter (Cin rounded up to 8); sub-filters per filter row
    int32_t in_bytes;          // size of `in` (below 2^31)
    int32_t tile_cfg;          // workgroup tile of the GEMM, see wino4_tile_m / _n
};
// Backward-weight of the same path: dy and x tiles transformed with the tile index as the
// GEMM depth, every GEMM tile cut into `split` >= 2 depth shares (slots), summed by the
// kernel that applies the final filter transform.
struct W4WgradArgs {
    const float *x, *dy;
    float *dw, *db;            // db nullable
    float *Wm, *Vm, *slots;    // workspace: transformed dy / x tiles, partial products [tile][split]
    float *D;                  // workspace: the 36 reduced products [pos][Kpad][Cpad]
    float *bias_part;          // workspace: [K][chunks*2], or null
    float scale;
    int32_t accumulate;
    int32_t N, C, H, W, K, P, Q, pad_h, pad_w;
    int32_t R, S, nsub, nsw;   // filter size (3..6), its 3x3 sub-filters, sub-filters per filter row
    int32_t TH, TW, T, chunks; // 4x4 output tiles per image (rows, cols), in total; 8-tile chunks of the depth
    int32_t Kpad, Cpad;        // rows of the two operands (Cpad: nsub * C rows q*C + c), multiples of the GEMM tile
    int32_t x_bytes, dy_bytes; // both below 2^31
    int32_t tile_cfg, split;
    FastDiv div_THW, div_TW;
};
hipError_t launch_wino4_wgrad(const W4WgradArgs &a, hipStream_t s);
int wino4_tile_m(int cfg);
int wino4_tile_n(int cfg);
hipError_t launch_wino4(const W4Args &a, hipStream_t s);
// The batched GEMM of that path on its own: C[b][m][n] = sum_d A[b][d][m] * B[b][d][n], A and
// B in MFMA order (depth/8, depth%2, row, (depth%8)/2, the last one contiguous), any number of
// batches b: the batch is the slowest part of the tile index.  `grid` workgroups take the tiles tile_base ...;
// with nsplit > 1 every tile is computed as nsplit depth shares into `slots`, which
// launch_w4_fixup adds up into C in a fixed order.
constexpr int kFftFreqs = 32 * 17;      // frequencies kept by the frequency-domain path: f = v * 17 + u, u < 17, v < 32
struct W4GemmArgs {
    const float *A, *B;
    float *C;
    float *slots;              // [tile][split] partial workgroup tiles of a launch with nsplit > 1
    int32_t chunks, Mpad, Npad, tiles_m, tiles_n;
    int32_t tile_base;         // first tile of this launch (tile order: row tile fastest, column tile, batch)
    int32_t nsplit;            // workgroups per tile, each taking an equal share of the chunks
    int32_t batch_inner;       // 0: A[b][chunk][half][row][4], C[b][row][col]; 1: A[chunk][half][b][row][4],
                               // C[row][b][col] with kFftFreqs batches (chunks * 2 * kFftFreqs * rows * 16 below 2^31)
};
void launch_w4_gemm(const W4GemmArgs &g, int cfg, unsigned grid, hipStream_t s);
void launch_w4_fixup(const W4GemmArgs &g, int cfg, unsigned tiles, hipStream_t s);

// Frequency-domain path for stride-1 layers whose padded input fits one 32 x 32 tile (see
// fft.hip): spectra of the images and filters, one complex product per frequency as a real
// GEMM with 2 x 2 blocks, inverse transform of the products.
struct FftArgs {                        // forward (mode 0) and backward-data (mode 1)
    const float *in;           // x, or dy
    const float *w;            // [K][C][R][S]
    const float *bias;         // nullable
    float *out;                // y, or dx
    float *A, *B, *M;          // workspace: image spectra (rows n), filter spectra (block form, columns
                               // 2 ch + po), products [f][Mpad][Npad]
    float *slots;
    int32_t split, split_tiles, tile_cfg;
    int32_t relu, mode;
    int32_t C;                 // channel count of w (its second axis)
    int32_t N, Cin, Hin, Win, Kout, Hout, Wout;
    int32_t in_off_h, in_off_w;    // where the image sits in its tile (the padding, or 0)
    int32_t out_off_h, out_off_w;  // where the output starts in the inverse tile (0, or the padding)
    int32_t R, S;
    int32_t chunks;            // 8-deep chunks of the 2*Cin-deep real product: ceil(Cin / 4)
    int32_t Mpad, Npad;        // N rows and 2*Kout columns, padded to the GEMM's workgroup tile
    int32_t in_bytes, w_bytes; // sizes of `in` and `w` (below 2^31)
};
hipError_t launch_fft_conv(const FftArgs &a, hipStream_t s);
struct FftWgradArgs {
    const float *x, *dy;
    float *dw, *db;            // db nullable
    float *A, *B, *M;          // workspace: spectra of dy (rows k), of x (conjugate block form, columns 2c+po), products
    float *slots;
    int32_t split, split_tiles, tile_cfg;
    float scale;
    int32_t accumulate;
    int32_t N, C, H, W, K, P, Q, R, S, pad_h, pad_w;
    int32_t chunks;            // ceil(N / 4): the images are the depth
    int32_t Mpad, Npad;        // K rows, 2*C columns, padded
    int32_t x_bytes, dy_bytes; // both below 2^31
};
hipError_t launch_fft_wgrad(const FftWgradArgs &a, hipStream_t s);

// Winograd backward-weight F(3x3,2x2) (see winograd_wgrad.hip).
struct WinoWgradArgs {
    const float *x;
    const float *dy;
    float *part;               // [splits][K][C][9]
    float *bias_part;          // [splits][K] partial sums of dy per filter, or null
    int32_t N, C, H, W, K, P, Q, pad_h, pad_w;
    int32_t TH, TW, T;         // 2x2 output tiles per image (rows, cols), in total; in the
                               // vector modes TW is rounded up to even (phantom last tile)
    int32_t mode;              // 0 per-element loads, 1 vector loads, 2 vector loads with
                               // an odd true tile-row width
    int32_t tiles_per_split;   // multiple of the 8-tile step
    int32_t tiles_k, tiles_c, splits;
    int32_t x_bytes, dy_bytes; // both below 2^31
    FastDiv div_THW, div_TW;
    // filters larger than 3x3 (per-element kernel only): tiles_c = nsub * tiles_c_sub
    // channel tiles; those of group q compute the 3x3 sub-filter gradient q from the
    // input shifted by (sub_dh[q], sub_dw[q]) and write it as channels q*C + c of part
    // [split][K][nsub*C][9].  nsub = 1: plain 3x3
    int32_t nsub, tiles_c_sub, sub_dh[4], sub_dw[4];
};

int wino_wgrad_tile();
int wino_wgrad_step();
hipError_t launch_wino_wgrad(const WinoWgradArgs &a, hipStream_t s);

// Direct backward-data for 3x3 stride-1 layers with C <= 4 (see direct_small.hip).
struct SmallCArgs {
    const float *dy;
    const float *w;
    float *dx;
    int32_t N, C, H, W, K, P, Q, pad_h;
    int32_t dy_bytes;
};
hipError_t launch_bwd_data_smallc(const SmallCArgs &a, hipStream_t s);

// ---------------------------------------------------------------------------
// Pointwise (1x1, stride 1, unpadded) layers as streaming products (see
// pointwise.hip).  out[n][r][p] = bias[r] + sum_d A[r][d] * in[n][d][p], p < HW.
// Forward: r = filter, d = input channel, A = w.  Backward-data: r = input channel,
// d = filter, A = w transposed.  A is element (r, d) at w[(r - r0[g]) * w_row_stride
// + d * w_depth_stride] of the group g that owns row r.
// ---------------------------------------------------------------------------
struct PwArgs {
    const float *in;
    int32_t in_bytes;                    // below 2^31
    int32_t out_bytes;                   // size of out[0] when ngroup == 1 (below 2^31)
    int32_t ngroup;                      // 1 .. kMaxGroups; rows r0[g] .. r0[g+1]-1 belong to group g
    const float *w[kMaxGroups];
    const float *bias[kMaxGroups];       // nullable
    float *out[kMaxGroups];              // group g: [N][r0[g+1]-r0[g]][HW]
    int32_t r0[kMaxGroups + 1];
    int32_t w_row_stride, w_depth_stride;
    int32_t depth_fast;                  // A's contiguous axis is the depth (forward) / the rows (backward-data);
                                         // stated, not derived from the strides: with one channel both are 1
    int32_t fill_vec;                    // A may be fetched as aligned 16-byte vectors along its contiguous axis
    int32_t wide_store;                  // set by the launcher: 16-byte stores through the LDS staging area
    int32_t relu;                        // forward: out = max(0, product + bias) (not with grouped outputs)
    int32_t D, Rout, HW, M;              // M = N*HW pixels
    int32_t ntiles;                      // 32-pixel tiles
    FastDiv div_HW, div_fast;            // div_fast: by D if depth_fast, else by Rout
    // taps form (launch_tap_stream): forward pass of an R x S layer; D = tC*tR*tS taps over a
    // tC x tH x tW input, HW = P*Q output pixels per image, tQ = Q
    int32_t tC, tH, tW, tR, tS, tsh, tsw, tph, tpw, tQ;
    int32_t tap_bwd;                     // stride-1 backward-data: in = dy, w walked as [k][c][r][t], taps flipped
    FastDiv div_tQ, div_tRS, div_rows;   // (the last two: tap_bwd fill, by tR*tS and by Rout)
};
hipError_t launch_tap_stream(const PwArgs &a, hipStream_t s);
// largest rows x depth product the kernel keeps in LDS, in bytes; 0 if the shape does not fit
size_t pw_stream_lds_bytes(int Rout, int D);
hipError_t launch_pw_stream(const PwArgs &a, hipStream_t s);

// Pointwise backward-weight: part[s][k][c] = sum over the pixels of range s of
// dy[n][k][p] * x[n][c][p]; bias_part[s][k] = the same sum of dy alone.  HW % 4 == 0,
// HW >= 16, both tensors below 2^31 bytes and 16-byte aligned, K <= 128, C <= 256.
struct PwWgradArgs {
    const float *x;
    const float *dy;
    float *part;               // [splits][K][C]
    float *bias_part;          // [splits][K], or null
    int32_t N, C, K, HW;
    int32_t x_bytes, dy_bytes;
    int32_t quads;             // N*HW/4 groups of 4 pixels
    int32_t steps_per_split;   // 16-pixel steps per split
    int32_t splits;
    int32_t tiles_c, phases;   // column groups x pixel phases = waves per workgroup (pw_wgrad_shape)
    FastDiv div_QW;            // by HW/4
    // taps form (launch_tap_wgrad): a small stride-1 R x S filter over xC channels of an
    // xH x xW image; C above is then the number of taps xC*R*S and HW = tP * Qd (dy plane)
    int32_t xC, xH, xW, tP, Qd, tR, tS, tph, tpw;
    FastDiv div_Q, div_RS, div_S;
};
hipError_t launch_tap_wgrad(const PwWgradArgs &a, hipStream_t s);
void pw_wgrad_shape(int C, int K, int HW, int *NJ, int *BT, int *PH);
hipError_t launch_pw_wgrad(const PwWgradArgs &a, hipStream_t s);

// Space-to-depth rearrangement of a strided layer's input (see space_to_depth.hip):
// x2[n][(a*s + b)*C + c][i][j] = x[n][c][s*i + a - pad_h][s*j + b - pad_w], channels
// s*s*C .. Cq-1 zero; x2 is N x Cq x H2 x W2.
struct S2dArgs {
    const float *x;            // space_to_depth: source
    float *x2;                 // space_to_depth: destination; depth_to_space: source
    float *dx;                 // depth_to_space: destination (shape of x)
    int32_t N, C, H, W, s, pad_h, pad_w, Cq, H2, W2;
    int32_t I2, J2;            // depth_to_space: (i, j) range covering all of dx
    FastDiv div_W2, div_J2;
};
hipError_t launch_space_to_depth(const S2dArgs &a, hipStream_t s);
hipError_t launch_depth_to_space(const S2dArgs &a, hipStream_t s);
// w [K][C][R][S] -> w2 [K][Cq][3][3], w2[k][(a*s + b)*C + c][r'][t'] = w[k][c][s*r' + a][s*t' + b]
hipError_t launch_filter_s2d(const float *w, float *w2, int K, int C, int R, int S, int stride, int Cq,
                             hipStream_t s);
// the inverse, dw = (dw +) the rearranged dw2
hipError_t launch_filter_d2s(const float *dw2, float *dw, int K, int C, int R, int S, int stride, int Cq,
                             int accumulate, hipStream_t s);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Opt-in kernel timing (see prof.hip): a ProfScope around the launch of a main kernel
// records a start and a stop event on the launch stream while conv2d_profile_begin is in
// effect, with the algorithmic flops and minimal bytes of the launch; otherwise it does
// nothing.
enum KernelId {
    KID_WINO4_GEMM = 0, KID_WINO4_INPUT, KID_WINO4_OUTPUT, KID_WINO4_WG_INPUT, KID_WINO4_WG_DY,
    KID_WINO_PAIR, KID_WINO_FUSED, KID_WINO_WGRAD_VEC, KID_WINO_WGRAD, KID_GEMMCONV, KID_WGRAD,
    KID_PW_STREAM, KID_PW_WGRAD, KID_SMALLC, KID_TAP_STREAM, KID_TAP_WGRAD, KID_FFT_IMAGE, KID_FFT_INVERSE, KID_FFT_FILTER, KID_COUNT
};
class ProfScope {
public:
    ProfScope(int kernel, double flops, double bytes, hipStream_t s);
    ~ProfScope();
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;
private:
    int slot_;
    hipStream_t stream_;
};

// Per-element operation y = fl(fl(a*x) + b) over n floats (see apply.hip).
hipError_t launch_apply_mul_add(const float *x, float *y, int64_t n, float a, float b, hipStream_t s);

}  // namespace mi355conv
