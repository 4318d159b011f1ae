// Stand-alone probe: the rate at which a gfx950 device retires back-to-back v_mfma_f32_32x32x16_bf16 (and, for
// comparison, v_mfma_f32_16x16x32_bf16) when nothing else runs, for all-zero and for random operands.  The published dense bf16 peak
// assumes the nominal clock; with random operands the device sustains visibly less, and that rate is the
// practical ceiling of the attention kernels.  Prints one line per case.
//
//   hipcc --offload-arch=gfx950 -O3 probe_mfma.hip -o probe_mfma && ./probe_mfma
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            std::fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                                 \
        }                                                                                 \
    } while (0)

// Eight MFMAs per loop trip on four independent accumulators; operands come from `src`.
__global__ __launch_bounds__(512) void mfma_loop(float *out, int trips, const float *src)
{
    f32x16 c[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) c[i][v] = 0.0f;
    bf16x8 a[8], b[8];
    for (int j = 0; j < 8; ++j)
        for (int e = 0; e < 8; ++e) {
            a[j][e] = (__bf16)src[(threadIdx.x * 64 + j * 8 + e) & 4095];
            b[j][e] = (__bf16)src[(threadIdx.x * 64 + 2048 + j * 8 + e) & 4095];
        }
    for (int r = 0; r < trips; ++r) {
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u], c[u & 3], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) s += c[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same with the 16x16x32 shape (half the flops per instruction, a quarter of the accumulator registers).
__global__ __launch_bounds__(512) void mfma_loop_16(float *out, int trips, const float *src)
{
    f32x4 c[8];
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 4; ++v) c[i][v] = 0.0f;
    bf16x8 a[8], b[8];
    for (int j = 0; j < 8; ++j)
        for (int e = 0; e < 8; ++e) {
            a[j][e] = (__bf16)src[(threadIdx.x * 64 + j * 8 + e) & 4095];
            b[j][e] = (__bf16)src[(threadIdx.x * 64 + 2048 + j * 8 + e) & 4095];
        }
    for (int r = 0; r < trips; ++r) {
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[u], c[u], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 4; ++v) s += c[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static void run16(float *out, const float *src, const char *what, int n_cu)
{
    const int nt = 512, trips = 80000;
    hipEvent_t t0, t1;
    CHECK(hipEventCreate(&t0));
    CHECK(hipEventCreate(&t1));
    hipLaunchKernelGGL(mfma_loop_16, dim3(n_cu), dim3(nt), 0, 0, out, 10, src);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(t0));
    hipLaunchKernelGGL(mfma_loop_16, dim3(n_cu), dim3(nt), 0, 0, out, trips, src);
    CHECK(hipEventRecord(t1));
    CHECK(hipDeviceSynchronize());
    float ms;
    CHECK(hipEventElapsedTime(&ms, t0, t1));
    const double flops = 2.0 * 16 * 16 * 32 * 8.0 * trips * (nt / 64) * n_cu;
    std::printf("%s operands, 16x16x32 shape, 2 wavefront(s) per SIMD: %.0f TFLOP/s\n", what, flops / (ms * 1e-3) / 1e12);
}

static void run(float *out, const float *src, const char *what, int n_cu)
{
    for (int waves_per_simd = 1; waves_per_simd <= 2; ++waves_per_simd) {
        const int nt = 256 * waves_per_simd, trips = 40000;
        hipEvent_t t0, t1;
        CHECK(hipEventCreate(&t0));
        CHECK(hipEventCreate(&t1));
        hipLaunchKernelGGL(mfma_loop, dim3(n_cu), dim3(nt), 0, 0, out, 10, src);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(t0));
        hipLaunchKernelGGL(mfma_loop, dim3(n_cu), dim3(nt), 0, 0, out, trips, src);
        CHECK(hipEventRecord(t1));
        CHECK(hipDeviceSynchronize());
        float ms;
        CHECK(hipEventElapsedTime(&ms, t0, t1));
        const double flops = 2.0 * 32 * 32 * 16 * 8.0 * trips * (nt / 64) * n_cu;
        std::printf("%s operands, %d wavefront(s) per SIMD: %.0f TFLOP/s\n", what, waves_per_simd, flops / (ms * 1e-3) / 1e12);
    }
}

int main()
{
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int n_cu = prop.multiProcessorCount;
    float *out, *zeros, *rnd;
    CHECK(hipMalloc(&out, (size_t)n_cu * 512 * 4));
    CHECK(hipMalloc(&zeros, 4096 * 4));
    CHECK(hipMalloc(&rnd, 4096 * 4));
    CHECK(hipMemset(zeros, 0, 4096 * 4));
    static float h[4096];
    std::srand(1);
    for (int i = 0; i < 4096; ++i) {            // sum of 12 uniforms - 6: approximately N(0, 1)
        float u = 0.0f;
        for (int j = 0; j < 12; ++j) u += std::rand() / (float)RAND_MAX;
        h[i] = u - 6.0f;
    }
    CHECK(hipMemcpy(rnd, h, sizeof(h), hipMemcpyHostToDevice));
    std::printf("%s, %d CUs, nominal clock %d MHz\n", prop.name, n_cu, prop.clockRate / 1000);
    run(out, zeros, "zero  ", n_cu);
    run(out, rnd, "random", n_cu);
    run16(out, zeros, "zero  ", n_cu);
    run16(out, rnd, "random", n_cu);
    return 0;
}
