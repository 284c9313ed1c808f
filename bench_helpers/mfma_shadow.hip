// What fits in the shadow of an int8 MFMA for a lone wave per SIMD?  The GEMM's main loop runs one
// wave per SIMD and places its other instructions between the MFMAs; this probe measures what that
// costs on this GPU: a register-only loop of v_mfma_i32_32x32x32_i8 (8 per iteration, 8 accumulator
// tiles) with n independent vector-ALU instructions, an LDS read or a global load (always the same
// cache lines: an L1 hit) placed after the MFMAs.  One workgroup of 4 waves per compute unit.
// Run by bench.py as a child process; prints one JSON line (nanoseconds per MFMA).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <cstdlib>

#define CK(x)                                                                                    \
    do {                                                                                         \
        hipError_t err_ = (x);                                                                   \
        if (err_ != hipSuccess) {                                                                \
            fprintf(stderr, "mfma_shadow: %s at line %d\n", hipGetErrorString(err_), __LINE__);  \
            exit(1);                                                                             \
        }                                                                                        \
    } while (0)

#define MFMA(A) "v_mfma_i32_32x32x32_i8 a[" A "], v[10:13], v[14:17], a[" A "]\n\t"
#define VALU2 "v_perm_b32 v20, v21, v22, v23\n\tv_perm_b32 v24, v25, v26, v27\n\t"
#define DSRD "ds_read_b128 v[28:31], v32\n\t"
#define GLD "global_load_dwordx4 v[36:39], v33, s[2:3]\n\t"
#define CLOB                                                                                              \
    "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v20", "v21", "v22", "v23", "v24", "v25",     \
    "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33", "v36", "v37", "v38", "v39", "s2", "s3", "s4", \
    "scc", "memory"
#define BODY(X)                                                                                         \
    MFMA("0:15") X MFMA("16:31") X MFMA("32:47") X MFMA("48:63") X MFMA("64:79") X MFMA("80:95") X      \
    MFMA("96:111") X MFMA("112:127") X

template <int MODE>
__global__ __launch_bounds__(256, 1) void probe(const uint8_t* src, long long* out, int iters) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[8192];
    const int tid = threadIdx.x;
    for (int i = tid; i < 2048; i += 256) reinterpret_cast<uint32_t*>(lds)[i] = i;
    __syncthreads();
    // every address stays inside lds[] (4 KB used) and inside the first MiB of src
    const uint32_t ldsaddr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds + (tid & 63) * 16 + (tid >> 6) * 1024;
    const uint32_t goff = (blockIdx.x * 256 + tid) * 16;
    const uint64_t base = reinterpret_cast<uint64_t>(src);
    const long long w0 = wall_clock64();
    asm volatile(
        "s_mov_b32 s2, %[blo]\n\t s_mov_b32 s3, %[bhi]\n\t"
        "v_mov_b32 v32, %[la]\n\t v_mov_b32 v33, %[go]\n\t"
        "v_mov_b32 v10, 0x01020304\n\t v_mov_b32 v11, 0x05060708\n\t v_mov_b32 v12, 0x11121314\n\t v_mov_b32 v13, 0x21222324\n\t"
        "v_mov_b32 v14, 0x01030507\n\t v_mov_b32 v15, 0x02040608\n\t v_mov_b32 v16, 0x0a0b0c0d\n\t v_mov_b32 v17, 0x1a1b1c1d\n\t"
        "v_mov_b32 v21, 1\n\t v_mov_b32 v22, 2\n\t v_mov_b32 v23, 0x03020100\n\t v_mov_b32 v25, 1\n\t v_mov_b32 v26, 2\n\t v_mov_b32 v27, 0x03020100\n\t"
        "s_mov_b32 s4, %[it]\n\t"
        "1:\n\t"
        : : [blo] "s"((uint32_t)base), [bhi] "s"((uint32_t)(base >> 32)), [la] "v"(ldsaddr), [go] "v"(goff), [it] "s"(iters)
        : CLOB);
    if (MODE == 0) asm volatile(BODY("") ::: CLOB);
    if (MODE == 1) asm volatile(BODY(VALU2) ::: CLOB);
    if (MODE == 2) asm volatile(BODY(VALU2 VALU2) ::: CLOB);
    if (MODE == 3) asm volatile(BODY(VALU2 VALU2 VALU2) ::: CLOB);
    if (MODE == 4) asm volatile(BODY(VALU2 VALU2 VALU2 VALU2) ::: CLOB);
    if (MODE == 5) asm volatile(BODY(DSRD) "s_waitcnt lgkmcnt(0)\n\t" ::: CLOB);
    if (MODE == 6)
        asm volatile(MFMA("0:15") GLD MFMA("16:31") MFMA("32:47") MFMA("48:63") MFMA("64:79") GLD MFMA("80:95")
                     MFMA("96:111") MFMA("112:127") "s_waitcnt vmcnt(4)\n\t" ::: CLOB);
    asm volatile(
        "s_sub_u32 s4, s4, 1\n\t s_cmp_lg_u32 s4, 0\n\t s_cbranch_scc1 1b\n\t s_waitcnt vmcnt(0) lgkmcnt(0)\n\t s_nop 15\n\t s_nop 15\n\t"
        ::: CLOB, "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15");
    const long long w1 = wall_clock64();
    if (tid == 0 && blockIdx.x == 0) out[0] = w1 - w0;
}

int main() {
    uint8_t* src;
    long long* out;
    CK(hipMalloc(&src, 2 << 20));
    CK(hipMemset(src, 1, 2 << 20));
    CK(hipMalloc(&out, 64));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount, iters = 20000;
    const char* names[] = {"mfma_only", "plus_2_valu", "plus_4_valu", "plus_6_valu", "plus_8_valu",
                           "plus_1_lds_read_b128", "plus_1_global_load_b128_per_4"};
    printf("{\"compute_units\": %d, \"mfmas\": %d, \"ns_per_mfma\": {", cus, iters * 8);
    for (int mode = 0; mode < 7; ++mode) {
        for (int rep = 0; rep < 2; ++rep) {
            switch (mode) {
#define L(M) case M: hipLaunchKernelGGL((probe<M>), dim3(cus), dim3(256), 0, 0, src, out, iters); break;
                L(0) L(1) L(2) L(3) L(4) L(5) L(6)
#undef L
            }
            CK(hipDeviceSynchronize());
        }
        long long ticks;
        CK(hipMemcpy(&ticks, out, 8, hipMemcpyDeviceToHost));
        printf("%s\"%s\": %.2f", mode ? ", " : "", names[mode], ticks * 10.0 / (iters * 8.0));   // 100 MHz ticks
    }
    printf("}}\n");
    CK(hipFree(src));
    CK(hipFree(out));
    return 0;
}
