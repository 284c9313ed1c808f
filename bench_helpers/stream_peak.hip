// Plain streaming kernels with the quantizer's memory access structure and none of its
// arithmetic: what the memory system of this GPU sustains for that structure.  Run by
// bench.py (as a child process) so that the quantizer's GB/s stands beside a measured
// ceiling as well as the 8 TB/s datasheet figure.
//
// Structure (as quantize_kernel): 512-thread workgroups, 4 x compute-unit-count of them,
// persistent; a wave takes a contiguous 4 KiB "super-chunk" (64 blocks of 32 bf16) per
// iteration as four 16-byte loads per lane, with the next super-chunk's loads issued as the
// registers free up.
//   read_only   loads only; the values are folded into one dword per lane, stored at the end
//   read_write  also the quantizer's stores: one dword per lane and pass (the codes) and two
//               64-byte runs of single bytes per super-chunk (exponent and dialect bytes)
// Sizes are the two streaming tensors of the benchmark; buffers rotate (6 inputs) so that
// no launch finds its input in the memory-side cache.  Prints one JSON line.
#include <hip/hip_runtime.h>
#include <chrono>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                                    \
    do {                                                                                         \
        hipError_t err_ = (x);                                                                   \
        if (err_ != hipSuccess) {                                                                \
            fprintf(stderr, "stream_peak: %s at line %d\n", hipGetErrorString(err_), __LINE__);  \
            exit(1);                                                                             \
        }                                                                                        \
    } while (0)

constexpr int kThreads = 512, kWaves = kThreads / 64;

template <bool WRITE>
__global__ __launch_bounds__(kThreads) void stream_kernel(const uint4* __restrict__ x, unsigned nsuper,
                                                          unsigned* __restrict__ codes,
                                                          unsigned char* __restrict__ eb,
                                                          unsigned char* __restrict__ db,
                                                          unsigned* __restrict__ sink) {
    const unsigned lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const unsigned stride = gridDim.x * kWaves;
    unsigned sc = blockIdx.x * kWaves + wave;
    uint4 w[4];
    if (sc < nsuper)
        for (int p = 0; p < 4; ++p) w[p] = x[(size_t)sc * 256u + p * 64 + lane];
    unsigned acc = 0;
    while (sc < nsuper) {
        const unsigned nsc = sc + stride;
        unsigned v[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            v[p] = w[p].x ^ w[p].y ^ w[p].z ^ w[p].w;
            if (WRITE) codes[(size_t)sc * 256u + p * 64 + lane] = v[p];
            if (nsc < nsuper) w[p] = x[(size_t)nsc * 256u + p * 64 + lane];
        }
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
        if (WRITE) {
            eb[(size_t)sc * 64u + lane] = (unsigned char)v[0];
            db[(size_t)sc * 64u + lane] = (unsigned char)v[1];
        }
        sc = nsc;
    }
    if (!WRITE) sink[blockIdx.x * kThreads + threadIdx.x] = acc;
}

template <bool WRITE>
static double median_ms(const std::vector<uint4*>& in, unsigned nsuper, unsigned grid, unsigned* codes,
                        unsigned char* eb, unsigned char* db, unsigned* sink) {
    const int n = 24;
    hipEvent_t e0[n], e1[n];
    for (int i = 0; i < n; ++i) {
        CK(hipEventCreate(&e0[i]));
        CK(hipEventCreate(&e1[i]));
    }
    // untimed load first: the clocks follow the load with a delay of some hundred milliseconds
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0; std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() < 120.0; ++i) {
        for (int j = 0; j < 32; ++j)
            hipLaunchKernelGGL(stream_kernel<WRITE>, dim3(grid), dim3(kThreads), 0, 0, in[(i * 32 + j) % in.size()], nsuper, codes, eb, db, sink);
        CK(hipDeviceSynchronize());
    }
    for (int i = 0; i < n; ++i) {
        CK(hipEventRecord(e0[i]));
        hipLaunchKernelGGL(stream_kernel<WRITE>, dim3(grid), dim3(kThreads), 0, 0, in[i % in.size()], nsuper, codes, eb, db, sink);
        CK(hipEventRecord(e1[i]));
    }
    CK(hipDeviceSynchronize());
    std::vector<float> ms(n);
    for (int i = 0; i < n; ++i) {
        CK(hipEventElapsedTime(&ms[i], e0[i], e1[i]));
        CK(hipEventDestroy(e0[i]));
        CK(hipEventDestroy(e1[i]));
    }
    std::sort(ms.begin(), ms.end());
    return ms[n / 2];
}

int main() {
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const unsigned grid = (unsigned)prop.multiProcessorCount * 4u;
    const long long shapes[2][2] = {{8192, 4096}, {4096, 14336}};
    printf("{\"compute_units\": %d", prop.multiProcessorCount);
    for (int s = 0; s < 2; ++s) {
        const size_t elems = (size_t)shapes[s][0] * shapes[s][1];
        const unsigned nsuper = (unsigned)(elems / 2048);            // 64 blocks of 32 per super-chunk
        std::vector<uint4*> in(6);
        for (auto& p : in) {
            CK(hipMalloc(&p, elems * 2));
            CK(hipMemset(p, 0x3c, elems * 2));
        }
        unsigned *codes, *sink;
        unsigned char *eb, *db;
        CK(hipMalloc(&codes, elems / 2));
        CK(hipMalloc(&eb, elems / 32));
        CK(hipMalloc(&db, elems / 32));
        CK(hipMalloc(&sink, (size_t)grid * kThreads * 4));
        const double ro = median_ms<false>(in, nsuper, grid, codes, eb, db, sink);
        const double rw = median_ms<true>(in, nsuper, grid, codes, eb, db, sink);
        const double rbytes = elems * 2.0, wbytes = elems * (0.5 + 2.0 / 32.0);
        printf(", \"%lldx%lld\": {\"read_only_ms\": %.4f, \"read_only_GBps\": %.1f, \"read_write_ms\": %.4f, "
               "\"read_write_GBps\": %.1f}",
               shapes[s][0], shapes[s][1], ro, rbytes / ro / 1e6, rw, (rbytes + wbytes) / rw / 1e6);
        for (auto& p : in) CK(hipFree(p));
        CK(hipFree(codes));
        CK(hipFree(eb));
        CK(hipFree(db));
        CK(hipFree(sink));
    }
    printf("}\n");
    return 0;
}
