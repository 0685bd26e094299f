// Prefill-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for M = eta * s prompt tokens (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the prefill phase is bound by FLOPs;
// Sec. 4.3: prefill micro-batch eta, prompt length s).
//
// One launch covers every linear of a stage that shares a storage variant: the launch's workgroups
// are the BM x 256 output tiles of all those linears, longest K first, so the chip stays full until
// the last few tiles instead of draining at the end of every linear.  The matrix instruction is
// v_mfma_f32_32x32x16_f16 (half the operand reads of 16x16x32 per multiply-accumulate).  Two kernels, chosen per storage
// variant (launch_tiles):
//
// prefill_kernel (3- and 4-bit codes; every variant at 128-token tiles): a workgroup of four wavefronts,
// one per SIMD with up to 512 registers per lane, computes a BM x 256 block of y.  Each wave owns one
// 64-row block of W (four 16-row tiles) for all BM tokens, so packed weight tiles go straight from
// global memory into that wave's registers in MFMA operand order, are dequantised there once per
// 128-column step (scale * code + zero, one fp16 rounding) and never touch LDS.  The activations
// of the block are shared by the four waves through a double-buffered LDS slab that is filled by
// direct global-to-LDS loads (no staging registers, no LDS store instructions); rows are 256 bytes
// apart and the 16-byte column index is XOR-ed with the row index, so the 16-byte operand reads
// of 16 consecutive token rows fall on 16 different bank groups.  Tiles t and t+2 of the wave's
// block make one 32-row operand, so a lane ends up with two consecutive output rows per token: 3/4-bit
// codes are loaded in that operand's lane order to begin with (a permutation of which lane fetches which
// 12 or 16 bytes), 8-bit codes and fp16 weights are paired with v_permlane16_swap after dequantisation.  The overlap of dequantisation, operand reads and
// matrix instructions is arranged inside each wave (see the main loop).
//
// prefill_ring_kernel (8-bit codes and fp16 weights at 256-token tiles): eight wavefronts, two per SIMD,
// both operands through a ring of LDS stages (described ahead of the kernel).
//
// On random operands either kernel runs the chip into its power limit (shader clock 1.45-1.7 GHz of a
// nominal 2.4 with the matrix pipe 60-70 % busy): what separates designs there is energy per
// multiply-accumulate -- bytes moved through LDS and from L2 -- more than idle issue slots.
#include <algorithm>
#include <mutex>
#include <type_traits>

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
            // opaque here, so that the widening to 64 bits happens next to the load and the instruction takes the
            // scalar base and the 32-bit lane offset as they are (no 64-bit vector add per load)
            asm volatile("" : "+v"(xoff[q]));
            __builtin_amdgcn_global_load_lds((gptr_t)(base + xoff[q]), (lptr_t)&sm.x[buf][row0][0], 16, 0, 0);
        }
    };
    // Packed weights of one 128-column step (3/4-bit codes) or of one 64-column half step (8-bit codes
    // and fp16 weights, whose tiles split into per-half pieces and are two to four times the size), as
    // loaded from global memory one (half) step ahead of their use.
    constexpr bool HALF_LOADS = (V == V_F16 || V == V_W8 || V == V_I8);
    struct WStep {
        WRaw<V> raw[NW];                             // HALF_LOADS: fp16 uses q[0], q[1]; 8-bit uses q[0]
        u32x2 s, z;                                  // fp16 scale / zero of the lane's four rows 4r..4r+3 (3/4-bit: [0] only, its two rows)
    };
    // 3/4-bit codes: a 32x32x16 B operand is tiles (p, p + 2) of the wave's block with lanes 0-15 / 16-31 on the two
    // tiles and lanes 32-63 two k slots further on.  Instead of loading each tile in its own lane order and exchanging
    // half the registers between lanes afterwards, a lane loads what it will hold: the packed codes of lane
    // r + 32 * khalf (+ 16 for the second operand) of tile p + 2 * sel, where r = lane % 16, sel = lane / 16 % 2,
    // khalf = lane / 32 -- the same bytes of the same tiles, in 192- or 256-byte runs per 16 lanes.  The lane's row of
    // the block is then 4 r + p + 2 sel for pair p.
    constexpr int TILE = VInfo<V>::TILE_BYTES, LANE_BYTES = TILE / 64;
    const int sel = (lane >> 4) & 1;
    uint32_t woff = (uint32_t)(2 * sel * TILE + LANE_BYTES * (r + 32 * (lane >> 5)));
    uint32_t soff = (uint32_t)(4 * r + 2 * sel) * 2u;
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
            // 3/4-bit codes arrive in the 32x32x16 operand's lane order (lane_src above): raw[p] is pair p's k slots
            // (kq 0, kq 2), raw[p + 2] its (kq 1, kq 3), 16 lanes further on in the tile.  Scalar base, 32-bit lane offset.
            const uint8_t* wbase = codes + ((size_t)rbc * KT + kt) * (4 * (size_t)TILE);
            asm volatile("" : "+v"(woff));
#pragma unroll
            for (int t = 0; t < NW; ++t) w.raw[t] = load_tile_at<V>(wbase + woff + (t & 1) * TILE + (t >> 1) * 16 * LANE_BYTES);
            if constexpr (SCHEME == SCH_ASYM) {      // rows 4r + 2 sel, 4r + 2 sel + 1: the lane's row of pair 0 and of pair 1
                const size_t row0 = ((size_t)kt * N + rbc * 64) * 2;
                asm volatile("" : "+v"(soff));
                w.s[0] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(scales) + row0 + soff);
                w.z[0] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(zeros) + row0 + soff);
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
                // 8-bit tiles keep their own lane order (tile t: row 4r + t); 3/4-bit operand t belongs to pair t & 1
                const uint32_t sp = w.s[HALF_LOADS ? t >> 1 : 0], zp = w.z[HALF_LOADS ? t >> 1 : 0];
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
    // step run from wb[h], the next half step is unpacked into wb[1 - h]: 3/4-bit codes a sixteenth of it
    // per segment (unpack_piece), the other variants one tile per segment in six of the segments.
    // Scheduling barriers keep the compiler from regrouping the segments.
    h8 wb[2][NW][2];
    WStep ws[2];                 // HALF_LOADS: raw half steps by parity; else this step's and the next step's codes
    auto unpack_tile = [&](const WStep& w, int t, int half, int dst) { operands(w, t, half, wb[dst][t]); };
    // 3/4-bit codes: a sixteenth of a half step's operands -- two pairs of codes of one operand, i.e. two registers:
    // piece idx = 4 * (operand t) + q covers pairs 2 q, 2 q + 1 of the operand's eight in this half.  One piece per
    // segment of four matrix instructions keeps the vector work between two of them under the 32 cycles the matrix
    // pipe takes for one (a wave on its own issues a vector instruction every 5-6 cycles).
    auto unpack_piece = [&](const WStep& w, int idx, int half, int dst) {
        if constexpr (!HALF_LOADS) {
            const int t = idx >> 2, q = idx & 3;
            const uint32_t sp = w.s[0], zp = w.z[0];
            const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
            const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
            const h2 s2 = splat(__builtin_bit_cast(_Float16, sh)), z2 = splat(__builtin_bit_cast(_Float16, zh));
#pragma unroll
            for (int k = 2 * q; k < 2 * q + 2; ++k) {
                const h2 c = __builtin_elementwise_fma(unpack_codes_pair<V>(w.raw[t], 8 * half + k), s2, z2);
                wb[dst][t][k >> 2][2 * (k & 3)] = c[0];
                wb[dst][t][k >> 2][2 * (k & 3) + 1] = c[1];
            }
        }
    };
    auto pair_tiles = [&](int p, int dst) {
        if constexpr (!HALF_LOADS) return;           // 3/4-bit codes were loaded in operand order
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
    // One 128-column step.  CUR: which of the two sets of packed weights holds this step's (the other receives the next
    // step's); the steps alternate, so that nothing is copied from one set to the other.
    auto step = [&](int kt, auto cur_set) {
        constexpr int CUR = HALF_LOADS ? 0 : decltype(cur_set)::value;
        const int buf = kt & 1;
        // Loads for the next step go out first and land while this step is multiplied.  Past the last
        // step they re-read it (no branches in the loop); what is built from them is never multiplied.
        const int ktn = min(kt + 1, kt_end - 1);
        if constexpr (!HALF_LOADS) load_w(ws[CUR ^ 1], ktn, 0);
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
            const WStep& src = HALF_LOADS ? ws[1 - half] : ws[CUR ^ half];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int mt = 0; mt < MTB; ++mt) {
                    const int seg = jj * MTB + mt, gseg = half * 2 * MTB + seg, cur = gseg & 1;
                    if (gseg + 1 < SEGS) {           // the next segment's activations (same slab)
                        // this segment's operands were read a segment ago: say so before the next reads go out, or the
                        // compiler (global-to-LDS loads in flight) waits for those too ahead of this segment's matrix instructions
                        __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
                        x_operands(buf, (gseg + 1) / MTB, (gseg + 1) % MTB, xa[cur ^ 1]);
                        // with no unpacking to place, the reads are best issued ahead of the segment's matrix instructions
                        if constexpr (V == V_F16) __builtin_amdgcn_sched_barrier(0);
                    }
                    acc[0][mt] = mfma32(xa[cur][0], wb[half][0][jj], acc[0][mt]);
                    acc[1][mt] = mfma32(xa[cur][0], wb[half][1][jj], acc[1][mt]);
                    acc[0][mt] = mfma32(xa[cur][1], wb[half][2][jj], acc[0][mt]);
                    acc[1][mt] = mfma32(xa[cur][1], wb[half][3][jj], acc[1][mt]);
                    if constexpr (HALF_LOADS) {
                        if (seg == 0 * STRIDE) unpack_tile(src, 0, 1 - half, 1 - half);
                        if (seg == 1 * STRIDE) unpack_tile(src, 2, 1 - half, 1 - half);
                        if (seg == 2 * STRIDE) pair_tiles(0, 1 - half);
                        if (seg == 3 * STRIDE) unpack_tile(src, 1, 1 - half, 1 - half);
                        if (seg == 4 * STRIDE) unpack_tile(src, 3, 1 - half, 1 - half);
                        if (seg == 5 * STRIDE) pair_tiles(1, 1 - half);
                    } else {
                        constexpr int PER_SEG = 16 / (2 * MTB);      // sixteen pieces over the half step's 2 * MTB segments
#pragma unroll
                        for (int i = 0; i < PER_SEG; ++i) unpack_piece(src, seg * PER_SEG + i, 1 - half, 1 - half);
                    }
                    if (half == 0 && (seg & 1) && seg < 2 * FILL_SEGS) fill_x_slab(ktn, buf ^ 1, (XQ / FILL_SEGS) * (seg >> 1), (XQ / FILL_SEGS) * ((seg >> 1) + 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): next slab written before anyone reads it
        __syncthreads();
    };
    int kt = kt_begin;
    for (; kt + 1 < kt_end; kt += 2) {
        step(kt, std::integral_constant<int, 0>());
        step(kt + 1, std::integral_constant<int, 1>());
    }
    if (kt < kt_end) step(kt, std::integral_constant<int, 0>());

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

// ---- 256-token tiles: eight waves, two per SIMD, both operands through LDS ------------------------------------
// A wave that issues in order stalls its SIMD's matrix pipe whenever it waits (an operand read, a memory wait, a
// barrier).  Here every SIMD holds two waves, so one wave's waits sit under the other's matrix instructions.  The
// workgroup computes a 256-token x 256-row block; wave (wm, wn) owns tokens 128 wm .. + 127 and the 64-row block wn
// (accumulators: 128 registers of the 256 a lane has at this occupancy).  Both operands come from LDS as fp16.
// The unit of work is a sub-step of 32 columns (a quarter of a quantisation group): sixteen matrix instructions
// per wave.
//   weights      a ring of four stages of one sub-step each: 16 tile pieces of 1 KB in the storage format's own lane
//                order (lane 16 kq + r: row r of the tile, columns 8 kq .. 8 kq + 7 of the 32).  A 32x32x16 B operand
//                is tiles (p, p + 2) of the wave's block read with lanes 0-15 / 16-31 on the two tiles: every 16 lanes
//                read 256 contiguous bytes.  fp16 weights are copied into place by global-to-LDS loads; packed codes
//                are loaded into registers, dequantised once per workgroup (wave w: tiles 2 w, 2 w + 1 of the
//                block's 16) and written with ds_write_b128.
//   activations  a ring of three stages of TWO sub-steps each, [256 tokens][64 columns]: rows of 128 bytes, so that a
//                fill takes whole 128-byte cache lines (with 64-byte rows every line is fetched from L2 twice, a
//                sub-step apart).  The 16-byte chunk c of row t is kept at position c ^ ((t >> 1) & 7): the operand
//                reads of 16 consecutive rows fall on 16 different bank groups.  Filled by global-to-LDS loads, eight
//                rows per instruction, half a stage per sub-step.
// One barrier per sub-step, B_i, placed ahead of sub-step i's matrix instructions, says two things: every wave's
// part of what sub-step i + 1 reads has landed (each waits for its own loads first), and every wave has finished
// sub-step i - 1, so what that sub-step read may be overwritten -- the weight stage with sub-step i + 3 right away;
// the activation stage, once both its sub-steps are done, with the columns of sub-steps i + 4 and i + 5.  Fills are
// so issued two to three sub-steps ahead of the barrier that needs them.  Because a sub-step's operands are
// published one barrier early, a wave reads the first operands of sub-step i + 1 while it multiplies the last of
// sub-step i, and the matrix instructions after a barrier start from registers.
constexpr int WRING = 4, XRING = 3;
struct PrefillRing {
    uint8_t x[XRING][32768];
    uint8_t w[WRING][16384];
};

// s_waitcnt immediate of gfx9: at most `vm` vector-memory and `lgkm` LDS / scalar-memory operations left in flight
// (as a builtin, so that the compiler's own wait insertion knows of it)
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (lgkm << 8); }

template <int V, bool SPLIT>
__global__ __launch_bounds__(512, 2)
void prefill_ring_kernel(const PrefillArgs a)
{
    int li = 0;
    while (li + 1 < a.n_lin && a.lin[li + 1].tile_begin <= (int)blockIdx.x) ++li;
    const PrefillLin& L = a.lin[li];
    const uint8_t* __restrict__ codes = L.codes;
    const uint16_t* __restrict__ scales = L.scales;
    const uint16_t* __restrict__ zeros = L.zeros;
    const uint16_t* __restrict__ bias = L.bias;
    uint16_t* y = L.y;                               // may alias L.residual
    const int M = a.M, K = L.K, N = L.N;
    constexpr int BM = 256;
    const int tile = (int)blockIdx.x - L.tile_begin;
    const int m_blocks = (M + BM - 1) / BM;
    const int per_xcd = SPLIT ? prefill_xcd_tiles(m_blocks, L.n_blocks, L.token_groups) : 0x7fffffff;
    const int split = SPLIT ? (tile >> 3) / per_xcd : 0;
    int tile_m, tile_n;
    if (!prefill_xcd_tile(m_blocks, L.n_blocks, L.token_groups, tile & 7, SPLIT ? (tile >> 3) % per_xcd : (tile >> 3), &tile_m, &tile_n)) return;
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr bool DMA_W = (V == V_F16);             // weights go to LDS as they are
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    PrefillRing& ring = *reinterpret_cast<PrefillRing*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int KT = K / 128;
    const int n_splits = SPLIT ? L.k_splits : 1;
    const int kt_share = KT / n_splits, kt_extra = KT % n_splits;
    const int kt_begin = split * kt_share + min(split, kt_extra), kt_end = kt_begin + kt_share + (split < kt_extra ? 1 : 0);
    const long RB = N / 64;
    const int m0 = tile_m * BM;
    const long rb = (long)tile_n * 4 + wn;           // the row block this wave multiplies
    const bool active = rb < RB;
    // sub-steps (32 columns) and double steps (64 columns) are counted from column 0 of the linear
    const int sub_begin = 4 * kt_begin, sub_last = 4 * kt_end - 1, dbl_last = sub_last >> 1;

    // ---- fills ------------------------------------------------------------------------------------------------
    // activations: instruction q = 4 wave + i of a stage covers token rows 8 q .. 8 q + 7; lane l fetches the chunk
    // that belongs at position l % 8 of row 8 q + l / 8.  Rows past M repeat row M - 1 (never stored).
    uint32_t xoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 8 * (4 * wave + i) + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        xoff[i] = ((uint32_t)min(row, M - 1 - m0) * (uint32_t)K + (uint32_t)c * 8u) * 2u;
    }
    const char* xtile = reinterpret_cast<const char*>(L.x + (size_t)m0 * K);
    auto fill_x = [&](int dbl, int xslot, int i) {   // double steps past the end repeat the last one (never multiplied)
        const char* base = xtile + (size_t)min(dbl, dbl_last) * 128;
        asm volatile("" : "+v"(xoff[i]));            // widened next to the load: scalar base + 32-bit lane offset, no 64-bit vector add
        __builtin_amdgcn_global_load_lds((gptr_t)(base + xoff[i]), (lptr_t)&ring.x[xslot][1024 * (4 * wave + i)], 16, 0, 0);
        asm volatile("" ::: "memory");
    };
    // weights: this wave brings tiles 2 wave, 2 wave + 1 of the block's 16 (row block wave / 2, tiles 2 (wave % 2), + 1)
    const long rb_fill = min((long)tile_n * 4 + (wave >> 1), RB - 1);
    const int t_fill = 2 * (wave & 1);
    const uint8_t* wsrc = codes + ((size_t)rb_fill * KT * 4 + t_fill) * (size_t)VInfo<V>::TILE_BYTES;     // + kt * 4 * TILE_BYTES
    uint32_t lane16[2] = {16u * (uint32_t)lane, 16u * (uint32_t)lane + 4096u};
    auto fill_w_dma = [&](int sub, int stage, int tt) {
        if constexpr (DMA_W) {
            const int sc = min(sub, sub_last);
            // scalar base + 32-bit lane offset (the second tile's 4096 bytes are beyond the instruction's immediate: they ride in the offset)
            const uint8_t* g = wsrc + (size_t)(sc >> 2) * 4 * 4096 + 1024 * (sc & 3);
            asm volatile("" : "+v"(lane16[tt]));
            __builtin_amdgcn_global_load_lds((gptr_t)(g + lane16[tt]), (lptr_t)&ring.w[stage][1024 * (2 * wave + tt)], 16, 0, 0);
            asm volatile("" ::: "memory");
        }
    };
    struct Packed {
        WRaw<V> t[2];
        u32x2 s, z;                                  // fp16 scale / zero of rows 4 r .. 4 r + 3 of the row block
    };
    const int r = lane & 15;
    auto load_packed = [&](Packed& pk, int kt) {
        if constexpr (!DMA_W) {
            const int ktc = min(kt, KT - 1);
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) pk.t[tt] = load_tile<V>(codes, rb_fill, KT, ktc, t_fill + tt, lane);
            if constexpr (SCHEME == SCH_ASYM) {
                const size_t idx = (size_t)ktc * N + rb_fill * 64 + 4 * r;
                pk.s = *reinterpret_cast<const u32x2*>(scales + idx);
                pk.z = *reinterpret_cast<const u32x2*>(zeros + idx);
            }
        }
    };
    // Two sets of packed codes: the group being turned into pieces and the one after it.  They swap roles with every
    // group (nothing is copied): ahead of a group's first piece the set that has just been used up receives the loads
    // of the group after next.
    Packed pk[2];
    auto rotate = [&](int piece, int kt_next, int free_set) {
        if constexpr (!DMA_W) {
            if (piece == 0) {
                load_packed(pk[free_set], kt_next);
                asm volatile("" ::: "memory");       // ahead of the sub-step's fills in issue order (see FILL_OPS)
            }
        }
    };
    // tile tt of piece `piece` of the group in set `set` -> stage
    auto produce = [&](int piece, int tt, int stage, int set) {
        if constexpr (!DMA_W) {
            const Packed& cur = pk[set];
            h8 v = unpack_codes_step<V>(cur.t[tt], piece);
            if constexpr (SCHEME == SCH_ASYM) {
                const int t = t_fill + tt;
                const uint32_t sp = (t >> 1) ? cur.s[1] : cur.s[0], zp = (t >> 1) ? cur.z[1] : cur.z[0];
                const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                const _Float16 sv = __builtin_bit_cast(_Float16, sh), zv = __builtin_bit_cast(_Float16, zh);
                const h8 s8 = {sv, sv, sv, sv, sv, sv, sv, sv}, z8 = {zv, zv, zv, zv, zv, zv, zv, zv};
                v = __builtin_elementwise_fma(v, s8, z8);
            }
            *reinterpret_cast<h8*>(&ring.w[stage][1024 * (2 * wave + tt) + 16 * lane]) = v;
        }
    };

    // ---- operand reads ----------------------------------------------------------------------------------------
    // A: token row 128 wm + 32 mt + l % 32, chunk 4 (sub-step's parity) + 2 slot + l / 32 (swizzled)
    // B: tiles (p, p + 2) of block wn
    uint32_t a_addr[2][2];
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int slot = 0; slot < 2; ++slot)
            a_addr[par][slot] = 128u * (uint32_t)(128 * wm + (lane & 31)) + 16u * (uint32_t)((4 * par + 2 * slot + (lane >> 5)) ^ ((lane >> 1) & 7));
    const uint32_t b_addr = 4096u * (uint32_t)wn + 2048u * (uint32_t)((lane >> 4) & 1) + 256u * (uint32_t)(lane >> 5) + 16u * (uint32_t)(lane & 15);
    struct Operands {
        h8 a[4], b[2];
    };
    auto read_operands = [&](Operands& o, int xslot, int par, int stage, int slot) {
        const uint8_t* xs = &ring.x[xslot][a_addr[par][slot]];
        const uint8_t* ws = &ring.w[stage][b_addr + 512 * slot];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) o.a[mt] = *reinterpret_cast<const h8*>(xs + 4096 * mt);
#pragma unroll
        for (int p = 0; p < 2; ++p) o.b[p] = *reinterpret_cast<const h8*>(ws + 1024 * p);
    };

    f16x acc[2][4];                                  // [tile pair (p, p + 2)][32-token tile]
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][mt][v] = 0.0f;
    auto multiply2 = [&](const Operands& o, int c) {       // two of a batch's eight matrix instructions
#pragma unroll
        for (int p = 0; p < 2; ++p) acc[p][c] = mfma32(o.a[c], o.b[p], acc[p][c]);
    };

    // Vector-memory instructions of one sub-step's fills, counted for the wait ahead of each barrier: B_i needs what
    // was issued up to sub-step i - 2, so the fills of sub-step i - 1 may stay in flight.  Loads of packed codes are
    // not counted: they are issued ahead of their sub-step's fills, so a wait that leaves only the newest FILL_OPS
    // operations in flight has waited for them too (never too little).
    constexpr int FILL_OPS = DMA_W ? 4 : 2;

    // ---- prologue: sub-steps 0 .. 2 of the weights, 0 .. 3 of the activations -----------------------------------
    load_packed(pk[0], kt_begin);
#pragma unroll
    for (int p = 0; p < WRING - 1; ++p) {
        rotate(p & 3, kt_begin + (p >> 2) + 1, 1);
        fill_w_dma(sub_begin + p, p, 0);
        fill_w_dma(sub_begin + p, p, 1);
        produce(p & 3, 0, p, 0);
        produce(p & 3, 1, p, 0);
    }
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int i = 0; i < 4; ++i) fill_x((sub_begin >> 1) + d, d, i);
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    Operands op[2];
    read_operands(op[0], 0, 0, 0, 0);
    static_assert(WRING == 4, "a group of four sub-steps is one turn of the weight ring: its stage is the sub-step's index in the group");
    int xc = 0;                                      // activation stage of the sub-step being multiplied
    // One group of four sub-steps.  SET: the set of packed codes that holds this group's (its last piece is produced in
    // the group's first sub-step; from the second on the pieces come from the next group, in the other set).
    auto group = [&](int kt, auto cur_set) {
        constexpr int SET = decltype(cur_set)::value;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(FILL_OPS, 0));
            __builtin_amdgcn_s_barrier();            // B_i
            asm volatile("" ::: "memory");
            const int sub = 4 * kt + j, par = j & 1;
            const int sc = j, sf = (j + WRING - 1) % WRING, sn = (j + 1) % WRING;      // this sub-step's weight stage, the free one, the next one
            const int xf = xc == 0 ? XRING - 1 : xc - 1, xn = xc == XRING - 1 ? 0 : xc + 1;      // (xc + 2) % 3 is free
            // the free weight stage takes sub-step i + 3: piece (j + 3) % 4 of group kt + (j + 3) / 4
            const int piece = (j + 3) & 3;
            // One batch of operand reads is in flight while the previous batch is multiplied (eight matrix
            // instructions, 256 cycles); the fills' memory instructions and the unpacking sit between the matrix
            // instructions, two apart.  Scheduling barriers keep that order.  The wait ahead of the second batch of
            // reads is free (the batch it waits for was issued a whole multiply earlier) and is there because the
            // compiler, with global-to-LDS loads in flight, waits for ALL outstanding LDS operations wherever it
            // needs one.
            read_operands(op[1], xc, par, sc, 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (c == 0) rotate(piece, kt + ((j + 3) >> 2) + 1, SET);
                if (c == 1) fill_x((sub + 4) >> 1, xf, 2 * par);
                if (c == 3) fill_x((sub + 4) >> 1, xf, 2 * par + 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply2(op[0], c);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
            read_operands(op[0], par ? xn : xc, par ^ 1, sn, 0);      // published by this sub-step's barrier
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (DMA_W) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (c == 1) fill_w_dma(sub + 3, sf, 0);
                    if (c == 3) fill_w_dma(sub + 3, sf, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply2(op[1], c);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // the unpacking of the two tiles (some forty vector instructions) is dealt out between the eight matrix
                // instructions: a long run of vector instructions from one wave keeps the other wave's matrix
                // instructions from issuing
                produce(piece, 0, sf, j == 0 ? SET : SET ^ 1);
                produce(piece, 1, sf, j == 0 ? SET : SET ^ 1);
#pragma unroll
                for (int c = 0; c < 4; ++c) multiply2(op[1], c);
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);       // a few vector instructions
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);       // an LDS write, if one is ready
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (par) xc = xn;
        }
    };
    int kt = kt_begin;
    for (; kt + 1 < kt_end; kt += 2) {
        group(kt, std::integral_constant<int, 0>());
        group(kt + 1, std::integral_constant<int, 1>());
    }
    if (kt < kt_end) group(kt, std::integral_constant<int, 0>());
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // the fills past the end have landed before the workgroup's LDS is released

    if (!active) return;
    // epilogue: lane (n = lane % 32, half = lane / 32) holds, for pair p, output row 64 rb + 4 (n % 16) + 2 (n / 16) + p
    // and tokens 128 wm + 32 mt + 8 (v / 4) + 4 half + v % 4: two consecutive rows per token -> 4-byte stores
    const int ncol = lane & 31, thalf = lane >> 5;
    const long nbase = rb * 64 + 4 * (ncol & 15) + 2 * (ncol >> 4);
    float post[2], bs[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        post[p] = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post[p] = (float)__builtin_bit_cast(_Float16, scales[nbase + p]);
        bs[p] = bias ? (float)__builtin_bit_cast(_Float16, bias[nbase + p]) : 0.0f;
    }
    if (SPLIT && L.k_splits > 1) {
        float* part = L.partial + (size_t)split * M * N;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tok = m0 + 128 * wm + 32 * mt + 8 * (v / 4) + 4 * thalf + (v % 4);
                if (tok >= M) continue;
                const f2 o = {acc[0][mt][v] * post[0], acc[1][mt][v] * post[1]};
                *reinterpret_cast<f2*>(part + (size_t)tok * N + nbase) = o;
            }
        return;
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tok = m0 + 128 * wm + 32 * mt + 8 * (v / 4) + 4 * thalf + (v % 4);
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
// Sets a kernel's dynamic-LDS limit once per device (the limit is a per-device property of the function).
template <typename F>
hipError_t allow_dynamic_lds(F* kernel, size_t bytes, std::once_flag* flags, hipError_t* results)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::call_once(flags[dev], [&] {
        results[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    });
    return results[dev];
}

template <int V, int BM>
hipError_t launch_tiles(const PrefillArgs& a, hipStream_t s)
{
    bool split = false;
    for (int li = 0; li < a.n_lin; ++li) split = split || a.lin[li].k_splits > 1;
    static std::once_flag flags[2][64];
    static hipError_t results[2][64];
    hipError_t e;
    // 256-token tiles: 3- and 4-bit codes go through the kernel that keeps the weights in registers (its unpacking is
    // hidden best there and it moves a third less through LDS; measured 2-6 % faster on OPT-30B-, 66B- and 176B-class
    // shapes), 8-bit codes and fp16 weights through the eight-wave kernel (3-20 % faster: their global loads are
    // four to eight times as large and stall a single wave per SIMD)
    if constexpr (BM == 256 && (V == V_W8 || V == V_I8 || V == V_F16)) {
        constexpr size_t smem = sizeof(PrefillRing);
        if (split) {
            if ((e = allow_dynamic_lds(&prefill_ring_kernel<V, true>, smem, flags[1], results[1])) != hipSuccess) return e;
            prefill_ring_kernel<V, true><<<(unsigned)a.total_tiles, 512, smem, s>>>(a);
        } else {
            if ((e = allow_dynamic_lds(&prefill_ring_kernel<V, false>, smem, flags[0], results[0])) != hipSuccess) return e;
            prefill_ring_kernel<V, false><<<(unsigned)a.total_tiles, 512, smem, s>>>(a);
        }
    } else {
        constexpr size_t smem = sizeof(PrefillSmem<BM>);
        if (split) {
            if ((e = allow_dynamic_lds(&prefill_kernel<V, BM, true>, smem, flags[1], results[1])) != hipSuccess) return e;
            prefill_kernel<V, BM, true><<<(unsigned)a.total_tiles, 256, smem, s>>>(a);
        } else {
            if ((e = allow_dynamic_lds(&prefill_kernel<V, BM, false>, smem, flags[0], results[0])) != hipSuccess) return e;
            prefill_kernel<V, BM, false><<<(unsigned)a.total_tiles, 256, smem, s>>>(a);
        }
    }
    e = hipGetLastError();
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
    return a.tokens_per_tile == 128 ? launch_tiles<V, 128>(a, s) : launch_tiles<V, 256>(a, s);
}

}  // namespace

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
