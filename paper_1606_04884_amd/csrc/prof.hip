// Opt-in timing of the library's main kernels with HIP events on the stream they are
// launched on (conv2d_profile_* in include/mi355conv.h), and two probes of what the chip
// sustains (a pure fp32 MFMA loop, a copy / fill stream) for calibrating roofline figures.
// Host-side state only; nothing here is on the path of a call while profiling is off.

#include "../../include/mi355conv.h"
#include "conv_internal.h"

#include <atomic>
#include <vector>

namespace mi355conv {

namespace {

struct ProfRec {
    int kernel;
    double flops, bytes;
};

std::atomic<int> g_prof_on{0};
std::atomic<int> g_prof_count{0};
int g_prof_capacity = 0;
std::vector<hipEvent_t> g_prof_events;      // 2 per record: start, stop
std::vector<ProfRec> g_prof_recs;

const char *const kKernelNames[KID_COUNT] = {
    "wino4_gemm_kernel", "wino4_input_kernel", "wino4_output_kernel", "wino4_wg_input_kernel",
    "wino4_wg_dy_kernel", "wino_pair_kernel", "wino_fused_kernel", "wino_wgrad_vec_kernel",
    "wino_wgrad_kernel", "gemmconv_kernel", "wgrad_kernel", "pw_stream_kernel",
    "pw_wgrad_kernel", "bwd_data_smallc_kernel", "pw_stream_kernel<TAPS>", "pw_wgrad_kernel<TAPS>",
    "fft_image_kernel", "fft_inverse_kernel", "fft_image_kernel<filters>",
};

}  // namespace

ProfScope::ProfScope(int kernel, double flops, double bytes, hipStream_t s) : slot_(-1), stream_(s)
{
    if (!g_prof_on.load(std::memory_order_relaxed)) return;
    const int i = g_prof_count.fetch_add(1);
    if (i >= g_prof_capacity) return;
    g_prof_recs[i] = {kernel, flops, bytes};
    if (hipEventRecord(g_prof_events[2 * i], s) == hipSuccess) slot_ = i;
}

ProfScope::~ProfScope()
{
    if (slot_ >= 0) (void)hipEventRecord(g_prof_events[2 * slot_ + 1], stream_);
}

// ---- probes ----------------------------------------------------------------
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// iters x 32 v_mfma_f32_32x32x2_f32 per wave on eight independent accumulators, nothing
// else in the loop; the result is stored so that the loop is kept
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(float *sink, int iters)
{
    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float a = (float)(threadIdx.x & 7) * 0.125f, b = (float)(threadIdx.x & 3) * 0.25f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 32; ++q) acc[q & 7] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q & 7], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) r += acc[i][0];
    if (r == 12345.678f) sink[0] = r;       // never true: keeps the accumulators live
}

// Copy / fill in the form that moved the most bytes in a sweep over grid sizes, loads in flight
// and cache hints on this chip: a workgroup takes spans of 4 x 256 vectors, all four loads issued
// before the first store, nontemporal hint on both sides (1 GiB: 6.0-6.2 TB/s read + write against
// 4.5-5.7 for one vector per thread and step; fill 5.9-6.0 TB/s when a workgroup writes one span).
// The vectors past the last whole span go one per thread.
__global__ __launch_bounds__(256) void probe_copy_kernel(const floatx4 *__restrict__ src, floatx4 *__restrict__ dst, int64_t n4)
{
    const int64_t spans = n4 / 1024;
    for (int64_t sp = blockIdx.x; sp < spans; sp += gridDim.x) {
        const int64_t i = sp * 1024 + threadIdx.x;
        const floatx4 v0 = __builtin_nontemporal_load(src + i), v1 = __builtin_nontemporal_load(src + i + 256);
        const floatx4 v2 = __builtin_nontemporal_load(src + i + 512), v3 = __builtin_nontemporal_load(src + i + 768);
        __builtin_nontemporal_store(v0, dst + i);
        __builtin_nontemporal_store(v1, dst + i + 256);
        __builtin_nontemporal_store(v2, dst + i + 512);
        __builtin_nontemporal_store(v3, dst + i + 768);
    }
    for (int64_t i = spans * 1024 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_fill_kernel(floatx4 *__restrict__ dst, int64_t n4, float v)
{
    const floatx4 x = {v, v, v, v};
    const int64_t spans = n4 / 1024;
    for (int64_t sp = blockIdx.x; sp < spans; sp += gridDim.x) {
        const int64_t i = sp * 1024 + threadIdx.x;
        dst[i] = x; dst[i + 256] = x; dst[i + 512] = x; dst[i + 768] = x;
    }
    for (int64_t i = spans * 1024 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) dst[i] = x;
}

}  // namespace mi355conv

using namespace mi355conv;

extern "C" {

int conv2d_profile_begin(int capacity)
{
    if (capacity < 1 || capacity > (1 << 20)) return CONV2D_ERR_GEOMETRY;
    g_prof_on.store(0);
    while ((int)g_prof_events.size() < 2 * capacity) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return CONV2D_ERR_LAUNCH;
        g_prof_events.push_back(e);
    }
    g_prof_recs.assign((size_t)capacity, ProfRec{0, 0.0, 0.0});
    g_prof_capacity = capacity;
    g_prof_count.store(0);
    g_prof_on.store(1);
    return CONV2D_OK;
}

int conv2d_profile_end(void)
{
    g_prof_on.store(0);
    const int n = g_prof_count.load();
    return n < g_prof_capacity ? n : g_prof_capacity;
}

int conv2d_profile_record(int i, int32_t *kernel, double *flops, double *bytes, float *ms)
{
    const int n = g_prof_count.load() < g_prof_capacity ? g_prof_count.load() : g_prof_capacity;
    if (i < 0 || i >= n) return CONV2D_ERR_GEOMETRY;
    if (!kernel || !flops || !bytes || !ms) return CONV2D_ERR_NULL;
    *kernel = g_prof_recs[i].kernel;
    *flops = g_prof_recs[i].flops;
    *bytes = g_prof_recs[i].bytes;
    if (hipEventElapsedTime(ms, g_prof_events[2 * i], g_prof_events[2 * i + 1]) != hipSuccess) return CONV2D_ERR_LAUNCH;
    return CONV2D_OK;
}

const char *conv2d_profile_kernel_name(int kernel)
{
    return kernel >= 0 && kernel < KID_COUNT ? kKernelNames[kernel] : "unknown";
}

int conv2d_probe_mfma_f32(float *sink, int32_t iters, double *flops, void *hip_stream)
{
    if (!sink || !flops) return CONV2D_ERR_NULL;
    if (iters < 1) return CONV2D_ERR_GEOMETRY;
    const int blocks = 512;                         // two workgroups of four waves per compute unit
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, sink, iters);
    *flops = (double)blocks * 4.0 * iters * 32.0 * (2.0 * 32 * 32 * 2);
    return hipGetLastError() == hipSuccess ? CONV2D_OK : CONV2D_ERR_LAUNCH;
}

int conv2d_probe_copy(const float *src, float *dst, int64_t n, void *hip_stream)
{
    if (!dst) return CONV2D_ERR_NULL;
    if (n < 4 || (n & 3) != 0 || (((uintptr_t)src | (uintptr_t)dst) & 15) != 0) return CONV2D_ERR_GEOMETRY;
    // grids the sweep found best: 16384 workgroups for the copy, one span per workgroup (up to
    // 65536) for the fill; at least one workgroup for the tail loop
    const int64_t spans = n / 4 / 1024;
    const int64_t cap = src ? 16384 : 65536;
    const int blocks = (int)(spans < 1 ? 1 : spans < cap ? spans : cap);
    if (src)
        hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream,
                           reinterpret_cast<const floatx4 *>(src), reinterpret_cast<floatx4 *>(dst), n / 4);
    else
        hipLaunchKernelGGL(probe_fill_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream,
                           reinterpret_cast<floatx4 *>(dst), n / 4, 1.0f);
    return hipGetLastError() == hipSuccess ? CONV2D_OK : CONV2D_ERR_LAUNCH;
}

}  // extern "C"
