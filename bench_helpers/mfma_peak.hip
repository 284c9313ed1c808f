// Register-only v_mfma_i32_32x32x32_i8 loop: what the int8 matrix cores of this GPU sustain
// with nothing else going on.  Run by bench.py (as a child process) to put the GEMM's
// throughput beside a measured peak as well as the datasheet one.  Three operand
// patterns, because the sustained clock depends on how many operand bits toggle:
// constants, uniformly random int8, random 4-bit magnitudes -- and, when a file is named
// as the second argument, operand bytes read from it (bench.py writes there a sample of
// the int8 operands the GEMM really multiplies: signed dialect magnitudes shifted by the
// block's exponent offset; 256 x 64 bytes of A operands followed by 256 x 64 bytes of W
// operands, one 64-byte slice per thread).  Prints one JSON line.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t err_ = (x);                                                                 \
        if (err_ != hipSuccess) {                                                              \
            fprintf(stderr, "mfma_peak: %s at line %d\n", hipGetErrorString(err_), __LINE__);  \
            exit(1);                                                                           \
        }                                                                                      \
    } while (0)

__device__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// 16 accumulator tiles (all 256 accumulation registers), 4 A and 4 B operand registers
__global__ __launch_bounds__(256) void mfma_loop(int* out, long long* clk, int iters, int mode, const int* operands) {
    v4i a[4], b[4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            const unsigned t = threadIdx.x * 64 + i * 8 + j;
            const unsigned mask = mode == 2 ? 0x0f0f0f0fu : 0xffffffffu;
            if (mode == 3) {
                a[i][j] = operands[threadIdx.x * 16 + i * 4 + j];
                b[i][j] = operands[4096 + threadIdx.x * 16 + i * 4 + j];
            } else {
                a[i][j] = mode ? (int)(mix(t) & mask) : 0x01010101;
                b[i][j] = mode ? (int)(mix(t + 77777) & mask) : 0x01010101;
            }
        }
    v16i acc[16];
    for (int i = 0; i < 16; ++i)
        for (int x = 0; x < 16; ++x) acc[i][x] = 0;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 16; ++i)
        for (int x = 0; x < 16; ++x) s += acc[i][x];
    const long long c1 = clock64(), w1 = wall_clock64();
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        clk[0] = c1 - c0;            // shader clocks
        clk[1] = w1 - w0;            // 100 MHz ticks
    }
}

int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 25000;
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int wgs = prop.multiProcessorCount;
    int* out;
    long long* clk;
    CK(hipMalloc(&out, (size_t)wgs * 256 * sizeof(int)));
    CK(hipMalloc(&clk, 64));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const char* names[4] = {"constant_operands", "random_int8_operands", "random_4bit_operands",
                            "sampled_gemm_operands"};
    // optional: 32 KiB of real operand bytes
    int* operands = nullptr;
    int nmodes = 3;
    if (argc > 2) {
        static int host[8192];
        FILE* f = fopen(argv[2], "rb");
        if (!f || fread(host, 1, sizeof(host), f) != sizeof(host)) {
            fprintf(stderr, "mfma_peak: cannot read 32768 operand bytes from %s\n", argv[2]);
            return 1;
        }
        fclose(f);
        CK(hipMalloc(&operands, sizeof(host)));
        CK(hipMemcpy(operands, host, sizeof(host), hipMemcpyHostToDevice));
        nmodes = 4;
    }
    printf("{\"compute_units\": %d, \"iters\": %d", wgs, iters);
    for (int mode = 0; mode < nmodes; ++mode) {
        float ms = 0;
        long long h[2] = {0, 1};
        for (int rep = 0; rep < 2; ++rep) {          // the second run is reported
            CK(hipEventRecord(e0));
            hipLaunchKernelGGL(mfma_loop, dim3(wgs), dim3(256), 0, 0, out, clk, iters, mode, operands);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            CK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
        }
        const double ops = 2.0 * 32 * 32 * 32 * 16 * (double)iters * 4.0 * wgs;
        printf(", \"%s\": {\"TOPs\": %.1f, \"MHz\": %.0f, \"clocks_per_mfma\": %.2f}", names[mode],
               ops / ms / 1e9, 100.0 * h[0] / h[1], (double)h[0] / (16.0 * iters));
    }
    printf("}\n");
    return 0;
}
