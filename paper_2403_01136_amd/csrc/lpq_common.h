// Host-side declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/lpq.h"

namespace lpq {

// One linear as the grouped kernels see it (passed by value in the kernel arguments).
struct LinDesc {
    const uint8_t* codes;
    const uint16_t* scales;
    const uint16_t* zeros;
    const uint16_t* x;      // fp16 [M][K]
    uint16_t* y;            // fp16 [M][N]
    const uint16_t* bias;   // fp16 [N] or null
    float* partial;         // split-K partial sums [ksplit][M][N] (null when ksplit == 1)
    int32_t K, N;
    int32_t variant;        // V_W3 .. V_F16
    int32_t ksplit;         // number of K ranges
    int32_t kt_per_split;   // 128-column tiles per K range
    int32_t row_blocks;     // N / rows per wave (64; 32 for fp16 weights)
    int32_t row_superblocks;// ceil(row_blocks / 4): one workgroup each
    int32_t unit_begin;     // first work unit (workgroup) of this linear in the launch
    int32_t red_begin;      // first reduction block of this linear (split-K only)
};

enum { MAX_LIN_PER_LAUNCH = 42 };   // keeps DecodeArgs under the 4 KB kernel-argument limit

struct DecodeArgs {
    int32_t n_lin, M, m0, total_units;   // m0: first token row of this pass (M > 64 is run 64 rows at a time)
    LinDesc lin[MAX_LIN_PER_LAUNCH];
};

// rows of W one decode wavefront covers, per variant (fp16 rows are 4x-16x bigger, so fewer of them)
__host__ __device__ inline int decode_rows_per_wave(int variant) { return variant == 4 ? 32 : 64; }

int variant_of(const lpq_qdesc& d);           // -1 if the (bits, scheme) pair is not supported
size_t tile_bytes_of(int variant);

// launchers (each returns a hipError_t from the launch)
hipError_t launch_quantize_pack(const void* w, const lpq_qdesc& d, const lpq_qweight& out, hipStream_t s);
hipError_t launch_unpack_dequant(const lpq_qweight& w, float* out, hipStream_t s);
hipError_t launch_decode(const DecodeArgs& a, int n_red_blocks, hipStream_t s);
hipError_t launch_prefill(const lpq_qweight& w, const void* x, int M, void* y, hipStream_t s);

}  // namespace lpq
