// Attainable rate of v_mfma_f32_32x32x16_bf16 on this chip, for reading the matrix-core fractions the benchmark
// reports (not part of the library: a stand-alone program).
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops mfma_rate_probe.hip -o mfma_rate_probe
//   ./mfma_rate_probe
//
// One wavefront per SIMD (256-thread workgroups that take 100 KB of LDS, so one workgroup per compute unit) runs a
// loop of matrix instructions over eight A and eight B operand registers per lane, with CH independent accumulators
// (CH = 1: every instruction depends on the one before).  Operands are either all 1.0 or random, roughly normal
// bf16 values: the data toggles the matrix pipes differently, and with it the power the chip draws and the clock it
// can hold.  Run on all 256 compute units and on 32.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define CHECK(x)                                                                   \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));         \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

template <int CH>
__global__ __launch_bounds__(256) void probe(const bf16x8* __restrict__ in, float* out, int iters) {
    bf16x8 a[8], b[8];
    for (int i = 0; i < 8; ++i) {
        a[i] = in[threadIdx.x * 16 + i];
        b[i] = in[threadIdx.x * 16 + 8 + i];
    }
    f32x16 acc[CH];
    for (int c = 0; c < CH; ++c) acc[c] = f32x16{};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int c = 0; c < CH; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b[(s + c) & 7], acc[c], 0, 0, 0);
    }
    float s = 0.f;
    for (int c = 0; c < CH; ++c)
        for (int v = 0; v < 16; ++v) s += acc[c][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int CH>
void run(const char* label, const bf16x8* in, int blocks, int iters) {
    float* out;
    CHECK(hipMalloc(&out, sizeof(float) * blocks * 256));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(probe<CH>), hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
    float ms = 0;
    for (int rep = 0; rep < 3; ++rep) {
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(probe<CH>, dim3(blocks), dim3(256), 100 * 1024, 0, in, out, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    const double n_mfma = (double)iters * 8 * CH;            // per wavefront = per SIMD
    const double flops = n_mfma * 32768.0 * blocks * 4;
    printf("%-8s chains %d  compute units %3d: %7.1f us, %5.2f ns per instruction and SIMD, %6.0f TFLOP/s\n", label, CH, blocks,
           ms * 1e3, ms * 1e6 / n_mfma, flops / (ms * 1e-3) / 1e12);
    CHECK(hipFree(out));
}

int main() {
    const int n = 256 * 16 * 8;
    std::vector<unsigned short> h(n);
    unsigned short *d_rand, *d_const;
    CHECK(hipMalloc(&d_rand, n * 2));
    CHECK(hipMalloc(&d_const, n * 2));
    srand(1);
    for (int i = 0; i < n; ++i) {   // roughly N(0,1): a sum of twelve uniforms, as bf16 bits
        float x = 0;
        for (int k = 0; k < 12; ++k) x += rand() / (float)RAND_MAX;
        x -= 6.f;
        unsigned u;
        memcpy(&u, &x, 4);
        h[i] = (unsigned short)(u >> 16);
    }
    CHECK(hipMemcpy(d_rand, h.data(), n * 2, hipMemcpyHostToDevice));
    for (int i = 0; i < n; ++i) h[i] = 0x3f80;   // 1.0
    CHECK(hipMemcpy(d_const, h.data(), n * 2, hipMemcpyHostToDevice));
    const int iters = 1000;
    for (int blocks : {256, 32}) {
        run<1>("ones", (const bf16x8*)d_const, blocks, iters);
        run<1>("random", (const bf16x8*)d_rand, blocks, iters);
        run<4>("ones", (const bf16x8*)d_const, blocks, iters);
        run<4>("random", (const bf16x8*)d_rand, blocks, iters);
    }
    return 0;
}
