// Host-side declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/lpq.h"

namespace lpq {

// One linear as the grouped decode kernels see it (passed by value in the kernel arguments).
// Its work is steps = row_superblocks * (K/128) "block steps" (one 128-column step of the
// WAVES row blocks a workgroup owns), each of weight `step_weight` (bytes streamed, scaled by a
// per-variant cost factor); `cum_weight` is the total weight of the linears before it.
// LinDesc::variant is the storage variant (0 .. 4: 3-, 4-, 8-bit grouped, 8-bit per row, fp16) -- or, in the descriptors
// of a stage-wide decode launch only, this: 3-bit codes that the kernel masks where they lie, against activations scaled
// for it beforehand (lpq_decode.hip); the host decides per launch.
enum { V_W3_INPLACE = 5 };

struct LinDesc {
    const uint8_t* codes;
    const uint16_t* scales;
    const uint16_t* zeros;
    const uint16_t* x;      // fp16 [M][K]
    uint16_t* y;            // fp16 [M][N]
    const uint16_t* bias;   // fp16 [N] or null
    const uint16_t* residual;   // fp16 [M][N] added to the output before its one rounding, or null
    uint64_t cum_weight;
    uint32_t step_weight;
    int32_t N;
    int32_t aux;            // stage-wide kernel: offset of the linear's prepared activations in DecodeArgs::prep, in 16-byte units;
                            // small-launch kernel: number of K splits
    uint16_t kt;            // K / 128 (K < 2^23)
    uint8_t variant;        // V_W3 .. V_F16, V_W3_INPLACE
    uint8_t act;            // lpq_activation applied to acc + bias (before the residual)
    __host__ __device__ int K() const { return (int)kt * 128; }
};
static_assert(sizeof(LinDesc) == 80, "48 of these and the header of DecodeArgs stay under 4 KB of kernel arguments");

enum { MAX_LIN_PER_LAUNCH = 48 };   // keeps DecodeArgs under 4 KB of kernel arguments (a stage of twelve layers in one launch)

// Even-share decomposition: the launch's total weight is cut into n_blocks equal ranges; workgroup
// b streams the steps whose start offset falls in [b, b+1) * total / n_blocks.  A (linear, row
// superblock) unit that a range boundary cuts is finished by the fix-up kernel from the fp32
// partial tiles the workgroups leave in `partial` (two slots per workgroup).
struct DecodeArgs {
    int32_t n_lin, M, m0, waves;         // m0: first token row of this pass (M > 64 is run 64 rows at a time)
    int32_t n_blocks, slot_floats;       // slot_floats: floats per partial tile = 64 tokens x rows per workgroup
    int32_t row_tiles, pad;              // small-launch kernel only: 16-row tiles per workgroup (2 .. 5; fp16 weights: at most 2)
    uint64_t total_weight;
    uint64_t range_q;                    // total_weight / n_blocks and
    uint32_t range_rem, pad2;            // total_weight % n_blocks: range b begins at range_q * b + range_rem * b / n_blocks
    float* partial;
    const uint16_t* prep;                // stage-wide kernel, up to 32 token rows per pass: what decode_prepare_kernel leaves
                                         // (the activations' group sums; for 3-bit weights the activations, scaled)
    LinDesc lin[MAX_LIN_PER_LAUNCH];
};
static_assert(sizeof(DecodeArgs) <= 4096, "kernel arguments are limited to 4 KB");

// One linear of a grouped prefill launch: its output is cut into tiles of BM tokens x 256 rows of W.
// Workgroup ids go round-robin over the chip's 8 XCDs (each with its own L2), so workgroup
// tile_begin + 8 * l + x is the l-th tile of XCD x (tile_begin is a multiple of 8).  The token blocks
// are split into token_groups groups and the row blocks into 8 / token_groups classes (row block n is
// in class n % classes); XCD x owns group x % token_groups and class x / token_groups and walks its
// tiles token block fastest, so the tiles an XCD runs at one time form a (token blocks) x (row blocks)
// rectangle whose activations and weights are fetched into that L2 once.  prefill_xcd_tile() decodes
// (x, l); 8 * prefill_xcd_tiles() workgroups cover the linear (those past an XCD's share exit).
struct PrefillLin {
    const uint8_t* codes;
    const uint16_t* scales;
    const uint16_t* zeros;
    const uint16_t* x;
    uint16_t* y;
    const uint16_t* bias;
    int32_t K, N;
    int32_t tile_begin;     // first tile (workgroup) of this linear in the launch
    int32_t n_blocks;       // ceil(N / 256)
    int32_t token_groups;   // 1, 2, 4 or 8
    int32_t act;            // lpq_activation applied to acc + bias (before the residual)
    const uint16_t* residual;   // fp16 [M][N] added to the output before its one rounding, or null
    // K split: with k_splits > 1 every tile is computed k_splits times over consecutive ranges of the
    // 128-column steps, each workgroup leaving its fp32 sums in partial[split][M][N]; a second kernel adds
    // the splits in order and applies bias, activation, residual and the one rounding.  An XCD's list of
    // tiles is then walked k_splits times (split-major), so the launch has k_splits times the workgroups.
    float* partial;
    int32_t k_splits, pad;
};

// Token block and row block of tile l of XCD x; false if that XCD has fewer tiles.
__host__ __device__ inline bool prefill_xcd_tile(int m_blocks, int n_blocks, int token_groups, int x, int l, int* tile_m, int* tile_n)
{
    const int classes = 8 / token_groups, tg = x % token_groups, rc = x / token_groups;
    const int group_size = (m_blocks + token_groups - 1) / token_groups;
    const int m_first = tg * group_size;
    const int m_cnt = m_blocks - m_first < group_size ? m_blocks - m_first : group_size;
    if (m_cnt <= 0) return false;
    *tile_m = m_first + l % m_cnt;
    *tile_n = rc + classes * (l / m_cnt);
    return *tile_n < n_blocks;
}

// Tiles of the busiest XCD.
__host__ __device__ inline int prefill_xcd_tiles(int m_blocks, int n_blocks, int token_groups)
{
    const int classes = 8 / token_groups;
    const int group_size = (m_blocks + token_groups - 1) / token_groups;      // group 0 is never smaller than the others
    const int rows_class0 = (n_blocks + classes - 1) / classes;               // nor is class 0
    return (group_size < m_blocks ? group_size : m_blocks) * rows_class0;
}

enum { MAX_PREFILL_LIN = 40 };   // keeps PrefillArgs under 4 KB of kernel arguments

struct PrefillArgs {
    int32_t n_lin, M, total_tiles;
    int32_t tokens_per_tile;       // 128 or 256
    PrefillLin lin[MAX_PREFILL_LIN];
};

// rows of W one decode wavefront covers, per variant (fp16 rows are 4x-16x bigger, so fewer of them)
__host__ __device__ inline int decode_rows_per_wave(int variant) { return variant == 4 ? 32 : 64; }
// stage-wide decode kernel: a wave's row blocks of a linear (N / rows per wave) and the workgroups' superblocks of them
__host__ __device__ inline int lin_row_blocks(const LinDesc& L) { return L.N >> (L.variant == 4 ? 5 : 6); }
__host__ __device__ inline int lin_row_superblocks(const LinDesc& L, int waves) { return (lin_row_blocks(L) + waves - 1) / waves; }
// small-launch decode kernel: 16-row tiles per workgroup (fp16 weights: at most two) and the groups of them in a linear
__host__ __device__ inline int rows_group_tiles(int variant, int row_tiles) { return (variant == 4 && row_tiles > 2) ? 2 : row_tiles; }
__host__ __device__ inline int rows_row_blocks(const LinDesc& L, int row_tiles) { return L.N / 16 / rows_group_tiles(L.variant, row_tiles); }

int variant_of(const lpq_qdesc& d);           // -1 if the (bits, scheme) pair is not supported
size_t tile_bytes_of(int variant);

// launchers (each returns a hipError_t from the launch)
// rows [row0, row0 + n_rows) of W (multiples of 64), read from a buffer that holds just those rows
hipError_t launch_quantize_pack(const void* w_rows, const lpq_qdesc& d, long row0, long n_rows, const lpq_qweight& out, hipStream_t s);
hipError_t launch_unpack_dequant(const lpq_qweight& w, float* out, hipStream_t s);
hipError_t launch_decode(const DecodeArgs& a, hipStream_t s);
// device address and size of the static scratch array of the current device (for the entry point that allocates nothing)
hipError_t static_scratch(void** ptr, size_t* bytes);
hipError_t launch_decode_rows(const DecodeArgs& a, hipStream_t s);     // small launches, M <= 32: cum_weight = workgroups before
hipError_t launch_prefill(int variant, const PrefillArgs& a, hipStream_t s);      // both kernels, if any linear is K-split
// variance indicator (lpq_indicator.hip)
size_t indicator_workspace_bytes(int N, long n8);
hipError_t launch_indicator(const void* w, int K, int N, const void* x, int M, int stochastic, double* omega, void* ws, hipStream_t s);
// the rest of the decoder layer (lpq_layer.hip)
hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, float eps, int M, int h, void* y, hipStream_t s);
int layernorm_max_hidden();
hipError_t launch_kv_append(const void* qkv, void* kc, void* vtc, int n_seqs, int T, int pos0, int H, int d, int S, hipStream_t s);
void attention_decode_plan(int n_seqs, int H, int L, int* range, int* splits);
size_t attention_decode_workspace_floats(int n_seqs, int H, int d, int splits);
hipError_t launch_attention(const void* qkv, const void* kc, const void* vtc, const float* slopes, int n_seqs, int T, int pos0, int H, int d,
                            int S, void* out, float* part, hipStream_t s);

}  // namespace lpq
