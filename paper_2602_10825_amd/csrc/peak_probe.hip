// Measured-achievable peaks on this GPU, to set beside the datasheet figures:
//   - bf16 matrix-core rate of a register-resident v_mfma_f32_32x32x16_bf16 loop, with
//     constant and with random operands (clocks are power-limited, so the data matter),
//   - HBM rate of a plain device copy and of a plain read.
// Stand-alone program (built next to the library); prints one line per measurement.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                             \
        }                                                                         \
    } while (0)

template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_loop(const bf16x8* in, float* out, long long* ticks, int iters) {
    const long long c0 = clock64(), w0 = wall_clock64();   // shader-clock and fixed-rate counters
    bf16x8 a[4], b[4];
    for (int j = 0; j < 4; ++j) {
        if (RANDOM) {
            a[j] = in[(threadIdx.x + 256 * j) * 2];
            b[j] = in[(threadIdx.x + 256 * j) * 2 + 1];
        } else {
            for (int i = 0; i < 8; ++i) { a[j][i] = (__bf16)1.0f; b[j][i] = (__bf16)0.5f; }
        }
    }
    f32x16 c[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], c[j], 0, 0, 0);
    }
    out[blockIdx.x * 256 + threadIdx.x] = c[0][0] + c[1][1] + c[2][2] + c[3][3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = clock64() - c0;
        ticks[1] = wall_clock64() - w0;
    }
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ s, uint4* __restrict__ d, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) d[i] = s[i];
}

__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ s, uint4* __restrict__ d, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const uint4 v = s[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) d[0] = acc;   // keeps the loads alive
}

int main() {
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    printf("device: %s, %d CUs, %d MHz\n", p.gcnArchName, p.multiProcessorCount, p.clockRate / 1000);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms;

    const int n16 = 1024 * 2 * 8;
    std::vector<unsigned short> h(n16);
    srand(1);
    for (int i = 0; i < n16; ++i) {
        const float f = ((rand() % 20001) - 10000) / 5000.0f;
        unsigned u;
        memcpy(&u, &f, 4);
        h[i] = (unsigned short)(u >> 16);
    }
    bf16x8* din;
    float* dout;
    CK(hipMalloc(&din, n16 * 2));
    CK(hipMemcpy(din, h.data(), n16 * 2, hipMemcpyHostToDevice));
    CK(hipMalloc(&dout, 512 * 256 * sizeof(float)));
    long long* dticks;
    CK(hipMalloc(&dticks, 16));
    int wall_khz = 0;
    CK(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, 0));
    // launch lengths from under 1 ms to tens of ms: the power limit acts over milliseconds, so
    // short launches run at higher clocks than a sustained kernel does
    const int lengths[4] = {5000, 25000, 100000, 400000};
    for (int mode = 0; mode < 2; ++mode) {
        for (int li = 0; li < 4; ++li) {
            const int iters = lengths[li];
            const double flops = 512.0 * 4 * (double)iters * 4 * 32768.0;
            for (int rep = 0; rep < 3; ++rep) {
                CK(hipEventRecord(e0));
                if (mode == 0) mfma_loop<false><<<512, 256>>>(din, dout, dticks, iters);
                else mfma_loop<true><<<512, 256>>>(din, dout, dticks, iters);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                CK(hipEventElapsedTime(&ms, e0, e1));
            }
            long long t[2];
            CK(hipMemcpy(t, dticks, 16, hipMemcpyDeviceToHost));
            printf("mfma_f32_32x32x16_bf16, %s operands, %7.2f ms launch: %.1f TFLOP/s, shader clock %.0f MHz\n",
                   mode ? "random" : "constant", ms, flops / ms / 1e9, (double)t[0] / (double)t[1] * wall_khz / 1e3);
        }
    }

    const size_t bytes = (size_t)2 << 30;
    uint4 *a, *b;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 1, bytes));
    CK(hipMemset(b, 2, bytes));
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        copy_kernel<<<8192, 256>>>(a, b, bytes / 16);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("device copy of 2 GiB: %.1f GB/s (read + write)\n", 2.0 * bytes / ms / 1e6);
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        read_kernel<<<2048, 256>>>(a, b, bytes / 16);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("device read of 2 GiB: %.1f GB/s\n", (double)bytes / ms / 1e6);
    CK(hipDeviceSynchronize());
    return 0;
}
