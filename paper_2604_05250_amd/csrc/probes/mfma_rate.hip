// Attainable rate of v_mfma_f32_32x32x16_bf16 on this GPU, as a function of the operand data.
//
// Stand-alone calibration program for the attention roofline (not part of the library): every compute
// unit runs four waves (one per SIMD) that issue nothing but this MFMA on register operands - no memory,
// no LDS, no other arithmetic - so the matrix cores are busy every cycle (32 cycles per instruction).
// What then varies with the operand data is the clock the chip sustains, hence the rate: the published
// dense bf16 peak assumes the maximum clock, which power management only grants for trivial operands.
//
// Build:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops mfma_rate.hip -o mfma_rate
// Run:    ./mfma_rate            (prints one line per operand distribution)
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                              \
    do {                                                                                      \
        hipError_t e_ = (x);                                                                  \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                    \
            return 1;                                                                         \
        }                                                                                     \
    } while (0)

constexpr int kMfmaPerIter = 32;

// 8 accumulators (accumulation VGPRs) x 4 A fragments x 4 B fragments, all in registers
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void mfma_loop(const intx4 *__restrict__ operands, float *out, long long *cycles, int iters)
{
    floatx16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    intx4 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[i * 256 + threadIdx.x];
        b[i] = operands[(4 + i) * 256 + threadIdx.x];
    }
    for (int i = 0; i < 8; ++i) asm volatile("" : "+a"(acc[i]));
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kMfmaPerIter; ++m)
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[m % 8]) : "v"(a[m % 4]), "v"(b[(m / 4) % 4]));
    }
    const long long t1 = __builtin_readcyclecounter();
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");      // the last results have landed
    float sum = 0.f;
    for (int i = 0; i < 8; ++i) {
        asm volatile("" : "+a"(acc[i]));
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    }
    out[blockIdx.x * 256 + threadIdx.x] = sum;
    if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
}

static uint16_t to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

int main()
{
    int dev = 0, cus = 0;
    CHECK(hipGetDevice(&dev));
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int n = 8 * 256 * 8;                        // bf16 values: 8 fragments x 256 lanes x 8 values
    std::vector<uint16_t> host(n);
    intx4 *operands;
    float *out;
    long long *cycles;
    CHECK(hipMalloc(&operands, n * 2));
    CHECK(hipMalloc(&out, (size_t)cus * 256 * 4));
    CHECK(hipMalloc(&cycles, (size_t)cus * 8));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const char *names[] = {"all zeros", "all 1.0", "A, B ~ N(0,1)", "A ~ N(0,1), B uniform in [0,1)",
                           "A ~ N(0,1), B = e^(-8u) (softmax-like weights)"};
    printf("%d compute units, 4 waves each, %d MFMAs per wave and launch\n", cus, 400 * kMfmaPerIter);
    for (int kind = 0; kind < 5; ++kind) {
        srand(1);
        for (int i = 0; i < n; ++i) {
            const float u1 = (rand() + 1.0f) / (RAND_MAX + 2.0f), u2 = (rand() + 1.0f) / (RAND_MAX + 2.0f);
            const float g = sqrtf(-2.f * logf(u1)) * cosf(6.2831853f * u2);
            const bool is_b = i / (256 * 8) >= 4;
            const float v = kind == 0 ? 0.f : kind == 1 ? 1.f : kind == 2 ? g : kind == 3 ? (is_b ? u1 : g)
                                                                              : (is_b ? expf(-8.f * u1) : g);
            host[i] = to_bf16(v);
        }
        CHECK(hipMemcpy(operands, host.data(), n * 2, hipMemcpyHostToDevice));
        const int iters = 400, launches = 20;
        for (int w = 0; w < launches; ++w) hipLaunchKernelGGL(mfma_loop, cus, 256, 0, 0, operands, out, cycles, iters);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        for (int w = 0; w < launches; ++w) hipLaunchKernelGGL(mfma_loop, cus, 256, 0, 0, operands, out, cycles, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipDeviceSynchronize());
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        std::vector<long long> hc(cus);
        CHECK(hipMemcpy(hc.data(), cycles, (size_t)cus * 8, hipMemcpyDeviceToHost));
        double avg = 0;
        for (int i = 0; i < cus; ++i) avg += (double)hc[i];
        avg /= cus;
        const double us = ms * 1e3 / launches, flops = (double)cus * 4 * iters * kMfmaPerIter * 32768.0;
        printf("%-48s %5.1f cycles per MFMA, %6.1f us per launch, %6.0f TFLOP/s, clock ~%.2f GHz\n", names[kind],
               avg / iters / kMfmaPerIter, us, flops / us / 1e6, avg / us / 1e3);
        fflush(stdout);
    }
    return 0;
}
