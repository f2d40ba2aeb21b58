// Measured denominators for the roofline figures: what this GPU sustains on an MFMA-only loop (bf16 and fp32)
// and on a plain device-to-device copy.  Not part of the conv1d library: a small library of its own
// (libconv1d_ubench.so) that the benchmark driver loads.  It allocates and frees its own buffers.
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// NACC independent accumulators per wave: enough to cover the MFMA latency, no memory traffic in the loop
template <int NACC>
__global__ __launch_bounds__(256) void mfma_bf16_32x32x16_kernel(float* out, int iters) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x + i) & 7));
        b[i] = static_cast<__bf16>(static_cast<float>(i));
    }
    f32x16 acc[NACC];
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void mfma_f32_32x32x2_kernel(float* out, int iters) {
    const float a = static_cast<float>(threadIdx.x & 7), b = 1.0f;
    f32x16 acc[NACC];
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// the 16 x 16 x 32 shape the bf16 kernels of the library use (4 accumulator registers per tile instead of 16)
template <int NACC>
__global__ __launch_bounds__(256) void mfma_bf16_16x16x32_kernel(float* out, int iters) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x + i) & 7));
        b[i] = static_cast<__bf16>(static_cast<float>(i));
    }
    typedef __attribute__((ext_vector_type(4))) float acc4;
    acc4 acc[NACC];
    for (int j = 0; j < NACC; ++j) acc[j] = acc4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        // (inline assembly with the accumulator tied to the destination: left to itself the compiler moves these small
        // accumulators between register files on every trip of the loop, and the loop then measures those moves)
        for (int j = 0; j < NACC; ++j) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(a), "v"(b));
    }
    float s = 0.f;
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 4; ++i) s += acc[j][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// the 16 x 16 x 4 shape the FP32 kernels of the library use (4 accumulator registers per tile instead of 16)
typedef __attribute__((ext_vector_type(4))) float f32x4;
template <int NACC>
__global__ __launch_bounds__(256) void mfma_f32_16x16x4_kernel(float* out, int iters) {
    const float a = static_cast<float>(threadIdx.x & 7), b = 1.0f;
    f32x4 acc[NACC];
    for (int j = 0; j < NACC; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(a), "v"(b));
    }
    float s = 0.f;
    for (int j = 0; j < NACC; ++j)
        for (int i = 0; i < 4; ++i) s += acc[j][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// write-only and read-only streams: a pass of the layer writes twice as many bytes as it reads, a copy does not
__global__ __launch_bounds__(256) void fill_kernel(float4* __restrict__ dst, size_t n) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    const float4 v{1.f, 2.f, 3.f, 4.f};
    for (; i < n; i += stride) dst[i] = v;
}

__global__ __launch_bounds__(256) void read_kernel(const float4* __restrict__ src, float* __restrict__ out, size_t n) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    float4 s{0.f, 0.f, 0.f, 0.f};
    for (; i < n; i += stride) {
        const float4 v = src[i];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    if (s.x + s.y + s.z + s.w == 12345.678f) out[0] = s.x;  // never true for the 0x01 pattern: keeps the loads alive
}

struct Timer {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok() { return hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~Timer() {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
    template <typename F>
    float best_ms(F launch, int reps) {
        launch();
        if (hipDeviceSynchronize() != hipSuccess) return -1.f;
        float best = -1.f;
        for (int r = 0; r < reps; ++r) {
            (void)hipEventRecord(e0, nullptr);
            launch();
            (void)hipEventRecord(e1, nullptr);
            if (hipEventSynchronize(e1) != hipSuccess) return -1.f;
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.f;
            if (best < 0.f || ms < best) best = ms;
        }
        return best;
    }
};

int num_cus() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return n;
}

}  // namespace

extern "C" {

// Sustained dense MFMA rate of the whole GPU in TFLOP/s with 2 waves per SIMD and no memory traffic.
// shape 0: v_mfma_f32_32x32x16_bf16, 1: v_mfma_f32_32x32x2_f32, 2: v_mfma_f32_16x16x4_f32 (same nominal rate as 1).
// Shapes 3-5 run ONE wave per SIMD, as the consumer waves of the library's kernels do: 3: 16x16x4 with 4 independent
// accumulators, 4: 16x16x4 with 8, 5: 32x32x2 with 4.  6: v_mfma_f32_16x16x32_bf16 with 2 waves per SIMD and 4 accumulators,
// 7: the same with one wave per SIMD and 8 accumulators, 8: one wave per SIMD and 13 accumulators.
// Returns 0 and writes *tflops, or -1 on a HIP error / unknown shape.
int conv1d_ubench_mfma_tflops(int shape, double* tflops) {
    const int ncu = num_cus();
    if (ncu <= 0 || !tflops) return -1;
    const int blocks = (shape >= 3 && shape != 6) ? ncu : ncu * 2, iters = 20000;  // 1 or 2 blocks of 4 waves per CU
    float* out = nullptr;
    if (hipMalloc(&out, static_cast<size_t>(blocks) * 256 * sizeof(float)) != hipSuccess) return -1;
    Timer t;
    float ms = -1.f;
    double flop = 0.0;
    if (t.ok()) {
        const double waves = static_cast<double>(blocks) * 4;
        switch (shape) {
            case 0:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_bf16_32x32x16_kernel<4>, dim3(blocks), dim3(256), 0, nullptr, out, iters); }, 3);
                flop = waves * iters * 4 * 2.0 * 32 * 32 * 16;
                break;
            case 1:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_f32_32x32x2_kernel<4>, dim3(blocks), dim3(256), 0, nullptr, out, iters / 4); }, 3);
                flop = waves * (iters / 4) * 4 * 2.0 * 32 * 32 * 2;
                break;
            case 2:
            case 3:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_f32_16x16x4_kernel<4>, dim3(blocks), dim3(256), 0, nullptr, out, iters); }, 3);
                flop = waves * iters * 4 * 2.0 * 16 * 16 * 4;
                break;
            case 4:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_f32_16x16x4_kernel<8>, dim3(blocks), dim3(256), 0, nullptr, out, iters / 2); }, 3);
                flop = waves * (iters / 2) * 8 * 2.0 * 16 * 16 * 4;
                break;
            case 5:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_f32_32x32x2_kernel<4>, dim3(blocks), dim3(256), 0, nullptr, out, iters / 4); }, 3);
                flop = waves * (iters / 4) * 4 * 2.0 * 32 * 32 * 2;
                break;
            case 6:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_bf16_16x16x32_kernel<4>, dim3(blocks), dim3(256), 0, nullptr, out, iters); }, 3);
                flop = waves * iters * 4 * 2.0 * 16 * 16 * 32;
                break;
            case 7:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_bf16_16x16x32_kernel<8>, dim3(blocks), dim3(256), 0, nullptr, out, iters); }, 3);
                flop = waves * iters * 8 * 2.0 * 16 * 16 * 32;
                break;
            case 8:
                ms = t.best_ms([&] { hipLaunchKernelGGL(mfma_bf16_16x16x32_kernel<13>, dim3(blocks), dim3(256), 0, nullptr, out, iters); }, 3);
                flop = waves * iters * 13 * 2.0 * 16 * 16 * 32;
                break;
            default: break;
        }
    }
    const bool launched = hipGetLastError() == hipSuccess;
    (void)hipFree(out);
    if (ms <= 0.f || !launched) return -1;
    *tflops = flop / (ms * 1e-3) / 1e12;
    return 0;
}

// Rate of a plain copy kernel over `bytes` of device memory (read + write counted, so 2 * bytes per pass) in GB/s.
// Sizes well above the 256 MB last-level cache measure HBM; small sizes measure that cache.
int conv1d_ubench_copy_gbps(size_t bytes, double* gbps) {
    const int ncu = num_cus();
    if (ncu <= 0 || !gbps || bytes < 4096) return -1;
    bytes &= ~static_cast<size_t>(15);
    float4 *a = nullptr, *b = nullptr;
    if (hipMalloc(&a, bytes) != hipSuccess) return -1;
    if (hipMalloc(&b, bytes) != hipSuccess) {
        (void)hipFree(a);
        return -1;
    }
    float ms = -1.f;
    Timer t;
    if (t.ok() && hipMemset(a, 1, bytes) == hipSuccess)
        ms = t.best_ms([&] { hipLaunchKernelGGL(copy_kernel, dim3(ncu * 8), dim3(256), 0, nullptr, a, b, bytes / 16); }, 5);
    const bool launched = hipGetLastError() == hipSuccess;
    (void)hipFree(a);
    (void)hipFree(b);
    if (ms <= 0.f || !launched) return -1;
    *gbps = 2.0 * static_cast<double>(bytes) / (ms * 1e-3) / 1e9;
    return 0;
}

// Rate of a write-only stream (mode 0) or a read-only stream (mode 1) over `bytes` of device memory in GB/s.
int conv1d_ubench_stream_gbps(int mode, size_t bytes, double* gbps) {
    const int ncu = num_cus();
    if (ncu <= 0 || !gbps || bytes < 4096 || (mode != 0 && mode != 1)) return -1;
    bytes &= ~static_cast<size_t>(15);
    float4* a = nullptr;
    float* out = nullptr;
    if (hipMalloc(&a, bytes) != hipSuccess) return -1;
    if (hipMalloc(&out, 256) != hipSuccess) {
        (void)hipFree(a);
        return -1;
    }
    float ms = -1.f;
    Timer t;
    if (t.ok() && hipMemset(a, 1, bytes) == hipSuccess) {
        if (mode == 0)
            ms = t.best_ms([&] { hipLaunchKernelGGL(fill_kernel, dim3(ncu * 8), dim3(256), 0, nullptr, a, bytes / 16); }, 5);
        else
            ms = t.best_ms([&] { hipLaunchKernelGGL(read_kernel, dim3(ncu * 8), dim3(256), 0, nullptr, a, out, bytes / 16); }, 5);
    }
    const bool launched = hipGetLastError() == hipSuccess;
    (void)hipFree(a);
    (void)hipFree(out);
    if (ms <= 0.f || !launched) return -1;
    *gbps = static_cast<double>(bytes) / (ms * 1e-3) / 1e9;
    return 0;
}

// Compute units and the nominal engine clock (MHz) the runtime reports for the current GPU.
int conv1d_ubench_device(int* compute_units, int* clock_mhz) {
    int dev = 0, khz = 0;
    if (!compute_units || !clock_mhz || hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) return -1;
    *compute_units = num_cus();
    *clock_mhz = khz / 1000;
    return 0;
}

}  // extern "C"
