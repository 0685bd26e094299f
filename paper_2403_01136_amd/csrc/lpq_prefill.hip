// Prefill-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for M = eta * s prompt tokens (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the prefill phase is bound by FLOPs;
// Sec. 4.3: prefill micro-batch eta, prompt length s).
//
// One launch covers every linear of a stage that shares a storage variant: the launch's workgroups
// are the BM x 256 output tiles of all those linears, longest K first, so the chip stays full until
// the last few tiles instead of draining at the end of every linear.
//
// A workgroup of four wavefronts computes a BM x 256 block of y.  Each wave owns one 64-row
// block of W (four 16-row tiles) for all BM tokens, so packed weight tiles go straight from
// global memory into that wave's registers in MFMA operand order, are dequantised there once per
// 128-column step (scale * code + zero, one fp16 rounding) and never touch LDS.  The activations
// of the block are shared by the four waves through a double-buffered LDS slab that is filled by
// direct global-to-LDS loads (no staging registers, no LDS store instructions); rows are 256 bytes
// apart and the 16-byte column index is XOR-ed with the row index, so the 16-byte operand reads
// of 16 consecutive token rows fall on 16 different bank groups.  The matrix instruction is
// v_mfma_f32_32x32x16_f16 (twice the rate of 16x16x32 on this chip): tiles t and t+2 of the wave's
// block are paired into 32-row operands with v_permlane16_swap after dequantisation, so a lane ends
// up with two consecutive output rows per token.  Registers are kept under 256
// per lane so that two workgroups share a CU and one's barrier and dequantisation overlap the
// other's matrix instructions.
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

template <int BM> struct PrefillSmem {
    uint16_t x[2][BM][128];        // [buffer][token row][column, 16-byte groups swizzled by row & 15]
};

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int V, int BM>
__global__ __launch_bounds__(256, BM > 128 ? 1 : 2)
void prefill_kernel(const PrefillArgs a)
{
    int li = 0;
    while (li + 1 < a.n_lin && a.lin[li + 1].tile_begin <= (int)blockIdx.x) ++li;
    const PrefillLin& L = a.lin[li];
    const uint8_t* __restrict__ codes = L.codes;
    const uint16_t* __restrict__ scales = L.scales;
    const uint16_t* __restrict__ zeros = L.zeros;
    const uint16_t* __restrict__ x = L.x;
    uint16_t* __restrict__ y = L.y;
    const uint16_t* __restrict__ bias = L.bias;
    const int M = a.M, K = L.K, N = L.N;
    // Tile order inside a linear: consecutive workgroup ids land on consecutive XCDs (8 of them, each
    // with its own L2), so workgroup id % 8 picks the token block within a group of 8 and id / 8 walks
    // the row blocks: every XCD then re-reads one token block's activations (which fit its L2) while
    // streaming different weights, instead of all XCDs sharing all token blocks.
    const int tile = (int)blockIdx.x - L.tile_begin;
    const int m_blocks = (M + BM - 1) / BM;
    int tile_m, tile_n;
    const int grouped = (m_blocks / 8) * 8 * L.n_blocks;         // tiles of the full groups of 8 token blocks
    if (tile < grouped) {
        const int g = tile / (8 * L.n_blocks), q = tile % (8 * L.n_blocks);
        tile_m = 8 * g + (q & 7);
        tile_n = q >> 3;
    } else {
        const int q = tile - grouped;
        tile_m = (m_blocks / 8) * 8 + q / L.n_blocks;
        tile_n = q % L.n_blocks;
    }
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr int NW = 4;                           // 16-row tiles per wave = one 64-row block
    constexpr int MTB = BM / 32;                    // 32-token tiles per block
    constexpr int XQ = BM / 16;                     // 1 KB global-to-LDS loads per wave and slab (4 rows each)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    PrefillSmem<BM>& sm = *reinterpret_cast<PrefillSmem<BM>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15;
    const int KT = K / 128;
    const long RB = N / 64;                          // 64-row blocks of W
    const int m0 = tile_m * BM;
    const long rb = (long)tile_n * 4 + wave;         // this wave's row block
    const bool active = rb < RB;                     // idle waves still stage activations
    const long rbc = active ? rb : RB - 1;

    f16x acc[2][MTB];                                // [tile pair (t, t+2)][token tile]
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][mt][v] = 0.0f;

    // slab fill: wave-load q of this wave covers token rows 4*(XQ*wave + q) .. +3; lane (row = lane/16,
    // slot = lane%16) fetches the 16-byte column group that belongs in that slot after swizzling.
    // Token rows past M are clamped to row M-1: they only feed outputs that are never stored.
    auto fill_x_slab = [&](int kt, int buf) {
#pragma unroll
        for (int q = 0; q < XQ; ++q) {
            const int row0 = 4 * (XQ * wave + q), row = row0 + (lane >> 4);
            const int c16 = (lane & 15) ^ (row & 15);
            const int tok = min(m0 + row, M - 1);
            const uint16_t* g = x + (size_t)tok * K + (size_t)kt * 128 + c16 * 8;
            __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)&sm.x[buf][row0][0], 16, 0, 0);
        }
    };
    // Packed weights of one 128-column step (3/4-bit codes) or of one 64-column half step (8-bit codes
    // and fp16 weights, whose tiles split into per-half pieces and are two to four times the size), as
    // loaded from global memory one (half) step ahead of their use.
    constexpr bool HALF_LOADS = (V == V_F16 || V == V_W8 || V == V_I8);
    struct WStep {
        WRaw<V> raw[NW];                             // HALF_LOADS: fp16 uses q[0], q[1]; 8-bit uses q[0]
        u32x2 s, z;                                  // fp16 scale / zero of the lane's four rows 4r..4r+3
    };
    auto load_w = [&](WStep& w, int kt, int half) {
        if constexpr (V == V_F16) {
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint8_t* tile = codes + (((size_t)rbc * KT + kt) * 4 + t) * 4096 + 2048 * half + 16 * lane;
                w.raw[t].q[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile));
                w.raw[t].q[1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 1024));
            }
        } else if constexpr (HALF_LOADS) {           // 8-bit: piece `half` of each tile
#pragma unroll
            for (int t = 0; t < NW; ++t) {
                const uint8_t* tile = codes + (((size_t)rbc * KT + kt) * 4 + t) * 2048 + 1024 * half + 16 * lane;
                w.raw[t].q[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile));
            }
            if constexpr (SCHEME == SCH_ASYM) {      // same group for both halves
                const size_t idx = (size_t)kt * N + rbc * 64 + 4 * r;
                w.s = *reinterpret_cast<const u32x2*>(scales + idx);
                w.z = *reinterpret_cast<const u32x2*>(zeros + idx);
            }
        } else {
#pragma unroll
            for (int t = 0; t < NW; ++t) w.raw[t] = load_tile<V>(codes, rbc, KT, kt, t, lane);
            if constexpr (SCHEME == SCH_ASYM) {
                const size_t idx = (size_t)kt * N + rbc * 64 + 4 * r;
                w.s = *reinterpret_cast<const u32x2*>(scales + idx);
                w.z = *reinterpret_cast<const u32x2*>(zeros + idx);
            }
        }
    };
    // MFMA operands of steps j = 2*half, 2*half + 1 of tile t (the unused half of the unpacking is dead code)
    auto operands = [&](const WStep& w, int t, int half, h8 out[2]) {
        if constexpr (V == V_F16) {
            out[0] = __builtin_bit_cast(h8, w.raw[t].q[0]);
            out[1] = __builtin_bit_cast(h8, w.raw[t].q[1]);
        } else {
            unpack_codes_half<V>(w.raw[t], half, out, 0);        // 8-bit pieces are loaded one at a time into q[0]
            if constexpr (SCHEME == SCH_ASYM) {
                const uint32_t sp = w.s[t >> 1], zp = w.z[t >> 1];
                const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                apply_scale_zero_half(out, __builtin_bit_cast(_Float16, sh), __builtin_bit_cast(_Float16, zh));
            }
        }
    };

    WStep wcur, wnext;
    load_w(wcur, 0, 0);
    fill_x_slab(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the slab (and the first weights) have landed
    __syncthreads();

    const int arow = lane & 31, ahalf = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        // start the next step's loads before anything else (weights first, the slab last, so that the
        // single wait before the barrier is also the wait the next step needs); they land while this
        // step's tiles are dequantised and multiplied
        if constexpr (!HALF_LOADS) { if (kt + 1 < KT) load_w(wnext, kt + 1, 0); }
        if (kt + 1 < KT) fill_x_slab(kt + 1, buf ^ 1);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if constexpr (HALF_LOADS) {
                if (half == 0) load_w(wnext, kt, 1);
                else if (kt + 1 < KT) load_w(wnext, kt + 1, 0);
            }
            // dequantise two steps of each tile, pair tiles (0,2) and (1,3) into 32-row operands:
            // wb[p] then covers k slots (kq 0, kq 2) and wb[p+2] slots (kq 1, kq 3)
            h8 wb[NW][2];
#pragma unroll
            for (int t = 0; t < NW; ++t) operands(wcur, t, half, wb[t]);
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) pair_tiles_for_mfma32(wb[p][jj], wb[p + 2][jj]);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = 2 * half + jj;
#pragma unroll
                for (int mt = 0; mt < MTB; ++mt) {
                    const int row = 32 * mt + arow;
                    const h8 a0 = *reinterpret_cast<const h8*>(&sm.x[buf][row][8 * ((4 * j + 2 * ahalf) ^ (row & 15))]);
                    const h8 a1 = *reinterpret_cast<const h8*>(&sm.x[buf][row][8 * ((4 * j + 2 * ahalf + 1) ^ (row & 15))]);
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        acc[p][mt] = mfma32(a0, wb[p][jj], acc[p][mt]);
                        acc[p][mt] = mfma32(a1, wb[p + 2][jj], acc[p][mt]);
                    }
                }
            }
            if constexpr (HALF_LOADS) {
                if (half == 0) { __builtin_amdgcn_s_waitcnt(0x0F70); wcur = wnext; }     // second half of this step
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): next slab written before anyone reads it
        __syncthreads();
        wcur = wnext;
    }

    if (!active) return;
    // epilogue: lane (n = lane%32, half = lane/32) holds, for pair p, output row 64*rb + 4*(n%16) + 2*(n/16) + p
    // and tokens 32*mt + 8*(v/4) + 4*half + v%4: two consecutive rows per token -> 4-byte stores
    const int ncol = lane & 31, thalf = lane >> 5;
    const long nbase = rb * 64 + 4 * (ncol & 15) + 2 * (ncol >> 4);
    float post[2], bs[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        post[p] = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post[p] = (float)__builtin_bit_cast(_Float16, scales[nbase + p]);
        bs[p] = bias ? (float)__builtin_bit_cast(_Float16, bias[nbase + p]) : 0.0f;
    }
#pragma unroll
    for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tok = m0 + 32 * mt + 8 * (v / 4) + 4 * thalf + (v % 4);
            if (tok >= M) continue;
            const h2 o = {(_Float16)(acc[0][mt][v] * post[0] + bs[0]), (_Float16)(acc[1][mt][v] * post[1] + bs[1])};
            *reinterpret_cast<h2*>(y + (size_t)tok * N + nbase) = o;
        }
}

// Tokens per tile.  Weight bytes are re-read from L2 once per token block, so the variants with the
// most bytes per weight (8-bit codes, fp16) take 256-token tiles (one workgroup per CU, 256
// accumulator registers); the others stay at 128 tokens and two workgroups per CU.
template <int V> struct PrefillTile { enum { BM = (V == V_W3 || V == V_W4) ? 128 : 256 }; };

template <int V>
hipError_t launch_variant(const PrefillArgs& a, hipStream_t s)
{
    constexpr int BM = PrefillTile<V>::BM;
    const size_t smem = sizeof(PrefillSmem<BM>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<V, BM>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    prefill_kernel<V, BM><<<(unsigned)a.total_tiles, 256, smem, s>>>(a);
    return hipGetLastError();
}

}  // namespace

int prefill_tokens_per_tile(int variant)
{
    switch (variant) {
    case V_W3: return PrefillTile<V_W3>::BM;
    case V_W4: return PrefillTile<V_W4>::BM;
    case V_W8: return PrefillTile<V_W8>::BM;
    case V_I8: return PrefillTile<V_I8>::BM;
    default: return PrefillTile<V_F16>::BM;
    }
}

hipError_t launch_prefill(int variant, const PrefillArgs& a, hipStream_t s)
{
    switch (variant) {
    case V_W3: return launch_variant<V_W3>(a, s);
    case V_W4: return launch_variant<V_W4>(a, s);
    case V_W8: return launch_variant<V_W8>(a, s);
    case V_I8: return launch_variant<V_I8>(a, s);
    case V_F16: return launch_variant<V_F16>(a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lpq
