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
// up with two consecutive output rows per token.  A workgroup has a CU to itself (one wave per SIMD,
// up to 512 registers per lane), so the overlap of dequantisation, operand reads and matrix
// instructions is arranged inside each wave (see the main loop).
#include <algorithm>

#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

template <int BM> struct PrefillSmem {
    uint16_t x[2][BM][128];        // [buffer][token row][column, 16-byte groups swizzled by row & 15]
};

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// SPLIT: some linear of the launch is K-split (the instantiation without it carries no second epilogue,
// whose registers the first would otherwise spill for).
template <int V, int BM, bool SPLIT>
__global__ __launch_bounds__(256, 1)
void prefill_kernel(const PrefillArgs a)
{
    int li = 0;
    while (li + 1 < a.n_lin && a.lin[li + 1].tile_begin <= (int)blockIdx.x) ++li;
    const PrefillLin& L = a.lin[li];
    const uint8_t* __restrict__ codes = L.codes;
    const uint16_t* __restrict__ scales = L.scales;
    const uint16_t* __restrict__ zeros = L.zeros;
    const uint16_t* __restrict__ x = L.x;
    uint16_t* y = L.y;                               // may alias L.residual
    const uint16_t* __restrict__ bias = L.bias;
    const int M = a.M, K = L.K, N = L.N;
    // Tile order inside a linear: workgroup ids go round-robin over the 8 XCDs; each XCD walks a
    // rectangle of token blocks x row blocks so that its L2 fetches those activations and weights once.
    const int tile = (int)blockIdx.x - L.tile_begin;
    const int m_blocks = (M + BM - 1) / BM;
    const int per_xcd = SPLIT ? prefill_xcd_tiles(m_blocks, L.n_blocks, L.token_groups) : 0x7fffffff;
    const int split = SPLIT ? (tile >> 3) / per_xcd : 0;         // 0 unless the linear is K-split
    int tile_m, tile_n;
    if (!prefill_xcd_tile(m_blocks, L.n_blocks, L.token_groups, tile & 7, SPLIT ? (tile >> 3) % per_xcd : (tile >> 3), &tile_m, &tile_n)) return;
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr int NW = 4;                           // 16-row tiles per wave = one 64-row block
    constexpr int MTB = BM / 32;                    // 32-token tiles per block
    constexpr int XQ = BM / 16;                     // 1 KB global-to-LDS loads per wave and slab (4 rows each)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    PrefillSmem<BM>& sm = *reinterpret_cast<PrefillSmem<BM>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: what derives from it (row block, LDS addresses of the slab loads) is then
    // scalar arithmetic instead of vector instructions in the main loop
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15;
    const int KT = K / 128;
    // this workgroup's 128-column steps: all of them, or the split's share (the first KT % k_splits splits take one more)
    const int n_splits = SPLIT ? L.k_splits : 1;
    const int kt_share = KT / n_splits, kt_extra = KT % n_splits;
    const int kt_begin = split * kt_share + min(split, kt_extra), kt_end = kt_begin + kt_share + (split < kt_extra ? 1 : 0);
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
    // The address of a load is a scalar base (start of the tile's rows, plus the step's columns) and a 32-bit
    // per-lane byte offset that does not change from step to step: (token row within the tile, clamped) * K + the
    // column group, kept in one register per load.
    uint32_t xoff[XQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int row = 4 * (XQ * wave + q) + (lane >> 4);
        const int c16 = (lane & 15) ^ (row & 15);
        xoff[q] = ((uint32_t)min(row, M - 1 - m0) * (uint32_t)K + (uint32_t)c16 * 8u) * 2u;
    }
    const char* xtile = reinterpret_cast<const char*>(x + (size_t)m0 * K);
    auto fill_x_slab = [&](int kt, int buf, int q_begin, int q_end) {
        const char* base = xtile + (size_t)kt * 256;
#pragma unroll
        for (int q = q_begin; q < q_end; ++q) {
            const int row0 = 4 * (XQ * wave + q);
            __builtin_amdgcn_global_load_lds((gptr_t)(base + xoff[q]), (lptr_t)&sm.x[buf][row0][0], 16, 0, 0);
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

    // Software pipeline inside the wave.  The matrix pipe runs one instruction at a time and a wave
    // issues in order, so vector work placed between two matrix instructions is free while work placed
    // in front of a run of them is not.  The step is therefore cut into segments of four matrix
    // instructions (one 32-token tile, both tile pairs, two k slots); while the segments of one half
    // step run from wb[h], the next half step is unpacked into wb[1 - h], one tile per segment.
    // Scheduling barriers keep the compiler from regrouping the segments.
    h8 wb[2][NW][2];
    WStep ws[2];                 // HALF_LOADS: raw half steps by parity; else this step's and the next step's codes
    auto unpack_tile = [&](const WStep& w, int t, int half, int dst) { operands(w, t, half, wb[dst][t]); };
    auto pair_tiles = [&](int p, int dst) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) pair_tiles_for_mfma32(wb[dst][p][jj], wb[dst][p + 2][jj]);
    };
    const int arow = lane & 31, ahalf = lane >> 5;
    auto x_operands = [&](int buf, int j, int mt, h8 out[2]) {
        const int row = 32 * mt + arow;
        out[0] = *reinterpret_cast<const h8*>(&sm.x[buf][row][8 * ((4 * j + 2 * ahalf) ^ (row & 15))]);
        out[1] = *reinterpret_cast<const h8*>(&sm.x[buf][row][8 * ((4 * j + 2 * ahalf + 1) ^ (row & 15))]);
    };

    load_w(ws[0], kt_begin, 0);
    if constexpr (HALF_LOADS) load_w(ws[1], kt_begin, 1);
    fill_x_slab(kt_begin, kt_begin & 1, 0, XQ);
#pragma unroll
    for (int t = 0; t < NW; ++t) unpack_tile(ws[0], t, 0, 0);
    pair_tiles(0, 0);
    pair_tiles(1, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the slab has landed
    __syncthreads();

    constexpr int SEGS = 4 * MTB;                    // segments per 128-column step
    constexpr int STRIDE = MTB / 4;                  // segments between two pieces of unpacking work
    constexpr int FILL_SEGS = 4;                     // odd segments that carry the next slab's loads
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const int buf = kt & 1;
        // Loads for the next step go out first and land while this step is multiplied.  Past the last
        // step they re-read it (no branches in the loop); what is built from them is never multiplied.
        const int ktn = min(kt + 1, kt_end - 1);
        if constexpr (!HALF_LOADS) load_w(ws[1], ktn, 0);
        // the next slab's 16 loads go out four at a time between the matrix instructions of the step's first
        // four odd segments (the even ones carry the unpacking): issued in a block up front they hold back
        // the step's first matrix instruction by as many issue slots, spread over more segments the last of
        // them land late (measured: 2, 4, 8 segments -> 4 is best)
        h8 xa[2][2];                                 // activations are read one segment ahead
        x_operands(buf, 0, 0, xa[0]);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if constexpr (HALF_LOADS) load_w(ws[half], ktn, half);       // the half step after next
            // the half step unpacked now: (kt, 1) during half 0, (kt + 1, 0) during half 1
            const WStep& src = HALF_LOADS ? ws[1 - half] : ws[half];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int mt = 0; mt < MTB; ++mt) {
                    const int seg = jj * MTB + mt, gseg = half * 2 * MTB + seg, cur = gseg & 1;
                    if (gseg + 1 < SEGS) {           // the next segment's activations (same slab)
                        x_operands(buf, (gseg + 1) / MTB, (gseg + 1) % MTB, xa[cur ^ 1]);
                        // with no unpacking to place, the reads are best issued ahead of the segment's matrix instructions
                        if constexpr (V == V_F16) __builtin_amdgcn_sched_barrier(0);
                    }
                    acc[0][mt] = mfma32(xa[cur][0], wb[half][0][jj], acc[0][mt]);
                    acc[1][mt] = mfma32(xa[cur][0], wb[half][1][jj], acc[1][mt]);
                    acc[0][mt] = mfma32(xa[cur][1], wb[half][2][jj], acc[0][mt]);
                    acc[1][mt] = mfma32(xa[cur][1], wb[half][3][jj], acc[1][mt]);
                    if (seg == 0 * STRIDE) unpack_tile(src, 0, 1 - half, 1 - half);
                    if (seg == 1 * STRIDE) unpack_tile(src, 2, 1 - half, 1 - half);
                    if (seg == 2 * STRIDE) pair_tiles(0, 1 - half);
                    if (seg == 3 * STRIDE) unpack_tile(src, 1, 1 - half, 1 - half);
                    if (seg == 4 * STRIDE) unpack_tile(src, 3, 1 - half, 1 - half);
                    if (seg == 5 * STRIDE) pair_tiles(1, 1 - half);
                    if (half == 0 && (seg & 1) && seg < 2 * FILL_SEGS) fill_x_slab(ktn, buf ^ 1, (XQ / FILL_SEGS) * (seg >> 1), (XQ / FILL_SEGS) * ((seg >> 1) + 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): next slab written before anyone reads it
        __syncthreads();
        if constexpr (!HALF_LOADS) ws[0] = ws[1];
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
    if (SPLIT && L.k_splits > 1) {                   // fp32 sums of this split; the reduce kernel finishes them
        float* part = L.partial + (size_t)split * M * N;
#pragma unroll
        for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tok = m0 + 32 * mt + 8 * (v / 4) + 4 * thalf + (v % 4);
                if (tok >= M) continue;
                const f2 o = {acc[0][mt][v] * post[0], acc[1][mt][v] * post[1]};
                *reinterpret_cast<f2*>(part + (size_t)tok * N + nbase) = o;
            }
        return;
    }
#pragma unroll
    for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tok = m0 + 32 * mt + 8 * (v / 4) + 4 * thalf + (v % 4);
            if (tok >= M) continue;
            float e0 = apply_activation(acc[0][mt][v] * post[0] + bs[0], L.act);
            float e1 = apply_activation(acc[1][mt][v] * post[1] + bs[1], L.act);
            if (L.residual) {
                const h2 res = *reinterpret_cast<const h2*>(L.residual + (size_t)tok * N + nbase);
                e0 += (float)res[0];
                e1 += (float)res[1];
            }
            const h2 o = {(_Float16)e0, (_Float16)e1};
            *reinterpret_cast<h2*>(y + (size_t)tok * N + nbase) = o;
        }
}

// Second kernel of a K-split linear: y = round(act(sum over splits + bias) + residual), four consecutive
// output rows of one token per thread, splits added in order (deterministic).
__global__ __launch_bounds__(256) void prefill_reduce_kernel(const PrefillArgs a, int li)
{
    const PrefillLin& L = a.lin[li];
    const size_t quads = (size_t)a.M * L.N / 4, plane = (size_t)a.M * L.N;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < quads; q += (size_t)gridDim.x * 256) {
        const size_t e = 4 * q;
        const int n = (int)(e % L.N);
        f4 sum = *reinterpret_cast<const f4*>(L.partial + e);
        for (int sp = 1; sp < L.k_splits; ++sp) sum += *reinterpret_cast<const f4*>(L.partial + sp * plane + e);
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        h4 res = {0, 0, 0, 0}, out;
        if (L.residual) res = *reinterpret_cast<const h4*>(L.residual + e);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float val = sum[v] + (L.bias ? (float)__builtin_bit_cast(_Float16, L.bias[n + v]) : 0.0f);
            val = apply_activation(val, L.act);
            if (L.residual) val += (float)res[v];
            out[v] = (_Float16)val;
        }
        *reinterpret_cast<h4*>(L.y + e) = out;
    }
}

// Tokens per tile: 256 (one workgroup per CU; 256 accumulator registers of the 512 a lane can have at one
// wave per SIMD).  Weight bytes are re-read from L2 once per token block and unpacked once per token block,
// so larger tiles mean fewer of both per matrix instruction.  A launch of at most 128 token rows has a single
// token block either way and takes 128-token tiles: half the matrix instructions per step.
template <int V, int BM>
hipError_t launch_tiles(const PrefillArgs& a, hipStream_t s)
{
    const size_t smem = sizeof(PrefillSmem<BM>);
    static bool attr_set = false;
    if (!attr_set) {
        for (const void* fn : {reinterpret_cast<const void*>(&prefill_kernel<V, BM, false>), reinterpret_cast<const void*>(&prefill_kernel<V, BM, true>)}) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    bool split = false;
    for (int li = 0; li < a.n_lin; ++li) split = split || a.lin[li].k_splits > 1;
    if (split) prefill_kernel<V, BM, true><<<(unsigned)a.total_tiles, 256, smem, s>>>(a);
    else       prefill_kernel<V, BM, false><<<(unsigned)a.total_tiles, 256, smem, s>>>(a);
    hipError_t e = hipGetLastError();
    for (int li = 0; li < a.n_lin && e == hipSuccess; ++li) {
        if (a.lin[li].k_splits <= 1) continue;
        const size_t quads = (size_t)a.M * a.lin[li].N / 4;
        const unsigned blocks = (unsigned)std::min<size_t>((quads + 255) / 256, 8192);
        prefill_reduce_kernel<<<blocks, 256, 0, s>>>(a, li);
        e = hipGetLastError();
    }
    return e;
}

template <int V>
hipError_t launch_variant(const PrefillArgs& a, hipStream_t s)
{
    return prefill_tokens_per_tile(V, a.M) == 128 ? launch_tiles<V, 128>(a, s) : launch_tiles<V, 256>(a, s);
}

}  // namespace

int prefill_tokens_per_tile(int /*variant*/, int M) { return M <= 128 ? 128 : 256; }

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
