// Issue-rate probe for gfx950 (MI355X): how many cycles of a SIMD a vector instruction of each kind costs at one to
// four wavefronts per SIMD, alone and next to matrix instructions, and what the instruction mix of one 3-bit decode
// step costs in different orders.  Not part of the library: a measuring tool for the design decisions recorded with
// the decode kernel (which instruction kinds are cheap, that matrix and two-operand vector instructions do not
// overlap, what a third and fourth wave per SIMD would buy).  Every kernel is a counted loop of register-only
// instructions; nothing is read or written but one guard store that never happens.
//
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 probe_issue_rates.hip -o probe_issue_rates && ./probe_issue_rates
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                             \
    do {                                                                                     \
        hipError_t e_ = (x);                                                                 \
        if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } \
    } while (0)

#define OPS(X)                                                       \
    X(0, "v_and_b32 %0, %0, %1")                                     \
    X(1, "v_lshrrev_b32 %0, 3, %0")                                  \
    X(2, "v_lshlrev_b32 %0, 3, %0")                                  \
    X(3, "v_mul_f32 %0, %1, %1")                                     \
    X(4, "v_fma_f32 %0, %1, %1, %0")                                 \
    X(5, "v_fma_mix_f32 %0, %1, %1, %0 op_sel_hi:[1,0,0]")           \
    X(6, "v_pk_fma_f16 %0, %1, %1, %0")                              \
    X(7, "v_perm_b32 %0, %0, %1, %1")                                \
    X(8, "v_and_or_b32 %0, %0, %1, %1")                              \
    X(9, "v_cvt_f32_f16 %0, %1")

static const char* op_names[] = {
#define X(N, S) S,
    OPS(X)
#undef X
};

#define MFMA(c) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b))

// 100 KB of LDS per workgroup: one workgroup per CU, so a workgroup of 256 * w threads is w waves per SIMD
#define PROLOGUE                                                                                           \
    h8 a, b;                                                                                               \
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)((threadIdx.x + i + seed) & 3); b[i] = (_Float16)((threadIdx.x * 3 + i) & 1); } \
    f4 c[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};                                    \
    uint32_t t[8];                                                                                         \
    for (int i = 0; i < 8; ++i) t[i] = threadIdx.x * 7 + i + seed;                                         \
    uint32_t kk = 0x3c003c00u;                                                                             \
    __shared__ uint32_t pad[25600];                                                                        \
    if (seed == 12345) pad[threadIdx.x] = seed;                                                            \
    __syncthreads();                                                                                       \
    const unsigned long long w0 = wall_clock64(), k0 = clock64();

#define EPILOGUE                                                                                           \
    const unsigned long long k1 = clock64(), w1 = wall_clock64();                                          \
    uint32_t s = 0;                                                                                        \
    for (int i = 0; i < 8; ++i) s ^= t[i];                                                                 \
    if (c[0][0] + c[1][1] + c[2][2] + c[3][3] + (float)s == 12345.678f) out[7] = s;                        \
    if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = k1 - k0; out[1] = w1 - w0; }

// 32 instructions of kind OP per iteration, with (MF) two matrix instructions among them
template <int OP, int MF>
__global__ void __launch_bounds__(1024) one_kind(unsigned long long* out, int iters, int seed)
{
    PROLOGUE
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (MF) MFMA(c[u]);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
#define X(N, S) if (OP == N) asm volatile(S : "+v"(t[v & 7]) : "v"(kk));
                OPS(X)
#undef X
            }
        }
    }
    EPILOGUE
}

#define AND(x) asm volatile("v_and_b32 %0, %0, %1" : "+v"(x) : "v"(kk))
#define SHR(x) asm volatile("v_lshrrev_b32 %0, 3, %0" : "+v"(x))
#define FMX(x) asm volatile("v_fma_mix_f32 %0, %1, %1, %0 op_sel_hi:[1,0,0]" : "+v"(x) : "v"(kk))

// One decode step of a wave at up to 16 token rows: 16 matrix instructions, SIMPLE shifts and masks, 16 fp32 FMAs.
// ORDER 0: a matrix instruction, then SIMPLE/16 shifts and masks, sixteen times; the FMAs at the end (the kernel's order)
// ORDER 1: the same with one FMA behind every matrix instruction
// ORDER 2: all matrix instructions first, then all vector work
// ORDER 3: the vector work alone;  ORDER 4: the matrix instructions alone
template <int ORDER, int SIMPLE>
__global__ void __launch_bounds__(1024) step_mix(unsigned long long* out, int iters, int seed)
{
    PROLOGUE
    constexpr int PER = SIMPLE / 16;
    for (int it = 0; it < iters; ++it) {
        if (ORDER == 0 || ORDER == 1) {
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                MFMA(c[m & 3]);
                if (ORDER == 1) FMX(t[m & 7]);
#pragma unroll
                for (int v = 0; v < PER; ++v) { if (v & 1) AND(t[v & 7]); else SHR(t[v & 7]); }
            }
            if (ORDER == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) FMX(t[v & 7]);
            }
        } else {
            if (ORDER == 2 || ORDER == 4) {
#pragma unroll
                for (int m = 0; m < 16; ++m) MFMA(c[m & 3]);
            }
            if (ORDER == 2 || ORDER == 3) {
#pragma unroll
                for (int v = 0; v < 16 * PER; ++v) { if (v & 1) AND(t[v & 7]); else SHR(t[v & 7]); }
#pragma unroll
                for (int v = 0; v < 16; ++v) FMX(t[v & 7]);
            }
        }
    }
    EPILOGUE
}

template <typename K>
static void time_kernel(K kernel, unsigned long long* out, int waves_per_simd, int iters, double* ns, double* ghz)
{
    const int threads = 256 * waves_per_simd;
    kernel<<<256, threads>>>(out, 200, 1);
    CHECK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    CHECK(hipEventRecord(e0));
    kernel<<<256, threads>>>(out, iters, 1);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    unsigned long long h[2];
    CHECK(hipMemcpy(h, out, 16, hipMemcpyDeviceToHost));
    *ns = ms * 1e6;
    *ghz = (double)h[0] / ((double)h[1] * 10.0);       // shader clock ticks / (100 MHz wall clock ticks x 10 ns)
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

template <int OP, int MF> static void run_one_kind(unsigned long long* out)
{
    const int iters = 20000;
    printf("%-48s %s", op_names[OP], MF ? "+mfma " : "      ");
    for (int w = 1; w <= 4; ++w) {
        double ns, ghz;
        time_kernel(one_kind<OP, MF>, out, w, iters, &ns, &ghz);
        printf("  %5.2f", ns / ((double)iters * 32.0 * w) * ghz);
    }
    printf("\n");
    fflush(stdout);
}

template <int ORDER, int SIMPLE> static void run_step_mix(const char* what, unsigned long long* out)
{
    const int iters = 5000;
    printf("%-54s", what);
    for (int w = 1; w <= 4; ++w) {
        double ns, ghz;
        time_kernel(step_mix<ORDER, SIMPLE>, out, w, iters, &ns, &ghz);
        printf("  %6.0f", ns / ((double)iters * w) * ghz);
    }
    printf("\n");
    fflush(stdout);
}

int main()
{
    unsigned long long* out;
    CHECK(hipMalloc(&out, 4096));
    printf("cycles of a SIMD per wave instruction (kernel time x shader clock / instructions issued on the SIMD), at 1 2 3 4 waves per SIMD;\n");
    printf("+mfma: one v_mfma_f32_16x16x32_f16 per 16 of them (its 16 pipe cycles included in the figure: 1.0 per instruction if nothing overlaps)\n");
#define X(N, S) run_one_kind<N, 0>(out);
    OPS(X)
#undef X
#define X(N, S) run_one_kind<N, 1>(out);
    OPS(X)
#undef X
    printf("\ncycles of a SIMD per decode step of one wave (16 matrix instructions, shifts and masks, 16 v_fma_mix_f32), at 1 2 3 4 waves per SIMD\n");
    run_step_mix<0, 128>("128 shifts and masks, kernel order", out);
    run_step_mix<0, 96>("96 shifts and masks (codes where they lie), kernel order", out);
    run_step_mix<1, 96>("96, an FMA behind every matrix instruction", out);
    run_step_mix<2, 96>("96, matrix instructions first, then vector work", out);
    run_step_mix<3, 96>("96, vector work alone", out);
    run_step_mix<4, 96>("matrix instructions alone", out);
    CHECK(hipFree(out));
    return 0;
}
