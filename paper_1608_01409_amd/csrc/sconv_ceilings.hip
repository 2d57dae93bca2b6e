// Ceilings microbenchmark for the sparse-convolution kernels on gfx950: the rates the roofline model and the
// tiling cost model take as machine parameters, measured the way the paper measures its machines with SGEMM
// and STREAM (Section 3.1).  Prints one line per figure.
//   v_fma_f32 rate            16 independent accumulators, SGPR multiplier
//   ds_read_b128 bandwidth    8 aligned reads in flight per wave
//   the inner loop's mix      4 v_fmac_f32 per ds_read_b128 (+ address add, + scalar work), see gen_ceilings.py
//   device copy bandwidth     float4 copy of 1 GiB; read alone and write alone over the same gigabyte
//   L2 read bandwidth         every workgroup reads the same 1 MiB over and over (it stays in each XCD's L2)
// All LDS addresses stay inside the 64 KB static array: lane*16 + (wave & 3)*1024 + offset (< 30.5 KB)
// + 2*1024 + 16.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 1;                                                                \
        }                                                                            \
    } while (0)

#include "sconv_ceilings_asm.inc"

constexpr double kClock = 2.4e9;
constexpr int kCUs = 256;

__global__ void __launch_bounds__(1024) k_fma(float *out, int iters)
{
    float a[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = threadIdx.x * 0.001f + i;
    const float b = threadIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
        const float sv = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(0x3f800000 + (it & 1)));
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) a[i] = fmaf(sv, b, a[i]);
    }
    float s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += a[i];
    if (s == 12345.678f) out[0] = s;
}

template <class V>
__global__ void __launch_bounds__(1024) k_mix(float *out, int iters)
{
    __shared__ float lds[16384];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) lds[i] = 1.0f;
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float r = V::run((unsigned)(lane * 16 + (wave & 3) * 1024), iters);
    if (r == 12345.678f) out[0] = r;
}

__global__ void __launch_bounds__(256) k_copy(const float4 *src, float4 *dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// sum of what is read, so the loads cannot be dropped; n float4s, grid-stride
__global__ void __launch_bounds__(256) k_read(const float4 *src, float *out, size_t n)
{
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float4 v = src[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) out[0] = acc.x;
}

__global__ void __launch_bounds__(256) k_write(float4 *dst, size_t n)
{
    const float4 v = make_float4(1.f, 2.f, 3.f, 4.f);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = v;
}

// every workgroup walks the same `n` float4s `reps` times: after the first pass they come from L2
__global__ void __launch_bounds__(256) k_read_l2(const float4 *src, float *out, int n, int reps)
{
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r = 0; r < reps; ++r)
        for (int i = threadIdx.x; i < n; i += 256) {
            const float4 v = src[(i + r * 64) % n];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) out[0] = acc.x;
}

template <class F>
static int time_ms(F launch, float *ms)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int i = 0; i < 5; ++i) {
        CK(hipEventRecord(e0));
        launch();
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float t;
        CK(hipEventElapsedTime(&t, e0, e1));
        if (t < best) best = t;
    }
    *ms = best;
    return 0;
}

template <class V>
static int run_mix(float *dout)
{
    const int iters = 2000;
    float ms;
    if (time_ms([&] { hipLaunchKernelGGL(k_mix<V>, dim3(kCUs), dim3(1024), 0, 0, dout, iters); }, &ms)) return 1;
    const double clk = ms * 1e-3 * kClock * kCUs;
    const double reads = (double)iters * V::kReadsPerIter * 16 * kCUs, fma = reads * V::kFmaPerRead * 64;
    printf("%-12s 16 waves/CU: %6.2f lanes-FMA/clk/CU (%5.1f%% of 64), LDS %6.1f B/clk/CU\n", V::name(), fma / clk,
           100 * fma / clk / 64, reads * 1024 / clk);
    return 0;
}

int main()
{
    float *dout;
    CK(hipMalloc(&dout, 1024));
    for (int thr : {512, 1024}) {
        const int iters = 20000;
        float ms;
        if (time_ms([&] { hipLaunchKernelGGL(k_fma, dim3(kCUs), dim3(thr), 0, 0, dout, iters); }, &ms)) return 1;
        const double fma = (double)kCUs * thr * iters * 64.0;
        printf("v_fma_f32    %2d waves/CU: %6.2f lanes-FMA/clk/CU, %.1f TFLOP/s at 2.4 GHz\n", thr / 64,
               fma / (ms * 1e-3) / kClock / kCUs, 2 * fma / ms / 1e9);
    }
#define X(V) if (run_mix<V>(dout)) return 1;
    SCONV_CEILING_VARIANTS(X)
#undef X
    const size_t bytes = (size_t)1 << 30;
    float4 *a, *b;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 1, bytes));
    float ms;
    if (time_ms([&] { hipLaunchKernelGGL(k_copy, dim3(kCUs * 8), dim3(256), 0, 0, a, b, bytes / 16); }, &ms)) return 1;
    printf("device copy  1 GiB: %.3f ms, %.2f TB/s (read + write)\n", ms, 2.0 * bytes / ms / 1e9);
    if (time_ms([&] { hipLaunchKernelGGL(k_read, dim3(kCUs * 8), dim3(256), 0, 0, a, dout, bytes / 16); }, &ms)) return 1;
    printf("HBM read     1 GiB: %.3f ms, %.2f TB/s\n", ms, 1.0 * bytes / ms / 1e9);
    if (time_ms([&] { hipLaunchKernelGGL(k_write, dim3(kCUs * 8), dim3(256), 0, 0, b, bytes / 16); }, &ms)) return 1;
    printf("HBM write    1 GiB: %.3f ms, %.2f TB/s\n", ms, 1.0 * bytes / ms / 1e9);
    {
        const int n = (1 << 20) / 16, reps = 64, wgs = kCUs * 8;
        if (time_ms([&] { hipLaunchKernelGGL(k_read_l2, dim3(wgs), dim3(256), 0, 0, a, dout, n, reps); }, &ms)) return 1;
        printf("L2 read      1 MiB per workgroup x %d, %d workgroups: %.3f ms, %.2f TB/s\n", reps, wgs, ms,
               (double)wgs * reps * (1 << 20) / ms / 1e9);
    }
    CK(hipFree(a));
    CK(hipFree(b));
    CK(hipFree(dout));
    return 0;
}
