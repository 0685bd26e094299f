// Decode-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for a small micro-batch M (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the decode phase is bound by the bytes it
// streams; Sec. 4.3: M = xi, one token per sequence).
//
// One grouped launch covers every linear of a stage, as one round of equally loaded workgroups.
// The launch's work is the list of (linear, 4 or 8 consecutive row blocks, 128-column step) items,
// each weighted by the bytes it streams; the list is cut into as many equal ranges as workgroups
// fit on the chip, and workgroup b streams range b.  Within a range a workgroup meets whole
// (linear, rows) units, which it finishes and stores as fp16, and at most two cut ones (its first
// and its last), whose fp32 partial tiles it leaves for a small fix-up kernel that adds the pieces
// of each cut unit in a fixed order (deterministic results).
//
// Inside a workgroup each wave owns one row block (64 rows of W; 32 for fp16 weights).  It streams
// its block's packed tiles from HBM as one sequential stream of 16-byte (12-byte for 3-bit)
// per-lane loads that are contiguous across the wave, keeps several 128-column steps in flight in
// registers, unpacks them there into MFMA B operands and multiplies them with the activations
// (MFMA A operands), which the workgroup stages once through a double-buffered LDS slab.
//
// Up to 32 token rows per pass the scale is applied after the matrix cores, per 128-column group, and the zero term
// (sum over groups of zero * sum of x) once per unit from the activations' group sums, which decode_prepare_kernel
// computes in front of the launch.
//
// A launch that streams little (a single linear of a decoder layer, up to 32 token rows per pass) takes a second
// kernel, decode_rows_kernel further down: one workgroup per group of 16-row tiles whose waves split K, no LDS
// staging, no fix-up pass.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

// RT: 16-row tiles per wave.  DEPTH: 128-column steps of weights a wave keeps in flight (a step is
// 3-4 KB per wave for 3/4-bit codes and 8 KB for 8-bit codes and fp16 rows, so 12-16 KB either way).
template <int V> struct DecodeCfg { enum { RT = (V == V_F16) ? 2 : 4, DEPTH = (V == V_W3 || V == V_W4) ? 4 : 2 }; };

// A launch is specialised on TOK, the token rows it covers: 16 or 32 (one or two 16-token tiles on the
// 16x16x32 MFMA, scale and zero applied after the matrix cores) or 64 (32x32x16 MFMA at twice the
// matrix-core rate, weights dequantised to fp16 in registers).  Activation staging: CHUNK 128-column steps per LDS
// buffer: at most CAP (8, or 16 where a launch of up to 16 token rows asks for it), and at most what lets two buffers
// of a workgroup fit 128 KB of the CU's LDS.
template <int TOK, int WAVES, int CAP> struct PipeCfg {
    enum { FIT = 32 * WAVES / TOK, CHUNK = FIT < CAP ? FIT : CAP };
    enum { ROW_HALVES = CHUNK * 128 };
    enum { XQ = TOK * CHUNK / 4 / WAVES };          // 1 KB global-to-LDS loads per wave and chunk
};

// Token row `row` keeps the 16-byte column group c16 of each of its 128-column steps in slot
// c16 ^ (row % 16) of that step: rows are a multiple of 256 bytes apart, and the swizzle makes the
// 16-byte operand reads of 16 consecutive rows hit 16 different bank groups.
template <int TOK, int WAVES, int CAP> struct DecodeSmem { uint16_t x[2][TOK][PipeCfg<TOK, WAVES, CAP>::ROW_HALVES]; };

// Halves per token row of a linear's group sums (see decode_prepare_kernel).
__device__ __host__ __forceinline__ int group_sums_stride(int K) { return 2 * ((K / 128 + 15) & ~15) + 8; }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// s_waitcnt vmcnt(N): all but the wave's newest N vector-memory operations have completed.  Also a
// compiler barrier, so that no memory operation moves across it.
template <int N> __device__ __forceinline__ void wait_vmem_all_but()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The codes of one MFMA step as fp16 subnormals, for the kernel that applies scale and zero after the matrix cores:
// 3-bit fields where they lie (the activations carry the inverse factors: 9 of a tile's 33 vector instructions less),
// wider ones moved to bit 0.  (4-bit fields in place save one instruction of six per register quadruple, less than
// preparing the activations costs: measured 0.3-4 % slower on 4-bit stages, so they are not.)
template <int V, bool INPL> __device__ __forceinline__ h8 unpack_post(const WRaw<V>& w, int j)
{
    if constexpr (V == V_W3 && INPL) return unpack_inplace_step<V>(w, j);
    else return unpack_subnormal_step<V>(w, j);
}

// A chunk: up to CHUNK consecutive 128-column steps of one (linear, row superblock) unit.
struct Chunk {
    int sb, kt0, n;      // row superblock, first step, number of steps (0 = none)
};

// The workgroup's share of one linear: block steps [s_begin, s_end) of L (step = sb * KT + kt), which
// may span several (linear, rows) units.  The weight pipeline runs on across unit boundaries; at
// the end of a unit the accumulators are stored -- as fp16 if the unit's whole K range lay inside
// [s_begin, s_end), else as an fp32 partial tile in slot_first (the unit this range entered mid-way)
// or slot_last (the unit it leaves mid-way) -- and cleared.
template <int V, int TOK, int WAVES, int CAP, bool INPL = false>
__device__ __forceinline__ void run_range(const LinDesc& L, int M, int m0, long s_begin, long s_end, const uint16_t* __restrict__ prep,
                                          float* __restrict__ slot_first, float* __restrict__ slot_last, DecodeSmem<TOK, WAVES, CAP>& sm)
{
    constexpr int RT = DecodeCfg<V>::RT;
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr bool WIDE = TOK > 32;                 // 32x32x16 path
    constexpr int MT = WIDE ? 1 : TOK / 16;         // narrow path: 16-token tiles
    constexpr int NP = RT / 2, MT2 = WIDE ? TOK / 32 : 1;      // wide path: tile pairs and 32-token tiles
    constexpr int CHUNK = PipeCfg<TOK, WAVES, CAP>::CHUNK, XQ = PipeCfg<TOK, WAVES, CAP>::XQ;
    // 32-token launches keep two steps in flight per wave: their second token tile needs the registers
    constexpr int WANT = TOK == 32 ? 2 : (int)DecodeCfg<V>::DEPTH;
    constexpr int STAGES = WANT < CHUNK ? WANT : CHUNK;
    // vector-memory loads of one Stage: the tiles (one load per KB, the 768-byte 3-bit tile included) and scale + zero
    constexpr bool POST = TOK <= 32 && V != V_F16;   // scale and zero folded in after the matrix cores (see compute below)
    constexpr bool INPLACE = POST && V == V_W3 && INPL;   // 3-bit codes masked where they lie, against activations scaled for it
    constexpr int STAGE_LOADS = RT * (VInfo<V>::TILE_BYTES >= 1024 ? VInfo<V>::TILE_BYTES / 1024 : 1) + (SCHEME == SCH_ASYM ? (POST ? 1 : 2) : 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int KT = L.kt;
    const int row_blocks = L.N / (V == V_F16 ? 32 : 64);     // of one wave each

    auto first_chunk = [&](long s) {
        Chunk c;
        c.sb = (int)(s / KT);
        c.kt0 = (int)(s % KT);
        c.n = (int)min((long)min(CHUNK, KT - c.kt0), s_end - s);
        return c;
    };
    auto next_chunk = [&](const Chunk& c) {
        Chunk d;
        d.sb = c.sb;
        d.kt0 = c.kt0 + c.n;
        if (d.kt0 == KT) { d.kt0 = 0; ++d.sb; }
        const long left = s_end - ((long)d.sb * KT + d.kt0);
        d.n = (c.n == 0 || left <= 0) ? 0 : (int)min((long)min(CHUNK, KT - d.kt0), left);
        return d;
    };
    // the wave's row block in a unit; waves past the end of W idle but still stage activations
    auto row_block = [&](int sb) { return (long)sb * WAVES + wave; };

    f4 acc[RT][MT];                   // narrow path
    f16x accw[NP][MT2];               // wide path: [tile pair][32-token tile]
    auto clear_acc = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < RT; ++t) acc[t][mt] = f4{0, 0, 0, 0};
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int m2 = 0; m2 < MT2; ++m2)
#pragma unroll
                for (int v = 0; v < 16; ++v) accw[p][m2][v] = 0.0f;
    };
    clear_acc();

    // ---- weight pipeline: one Stage = everything one 128-column step needs from global memory
    struct Stage {
        WRaw<V> w[RT];
        u32x2 s, z;          // fp16 scale / zero of the lane's four rows (tiles 0..3), grouped scheme only (z: 64-token path only)
    };
    Stage st[STAGES];
    // A load's address is a scalar base -- the workgroup's first row block of superblock sb at step kt -- plus a 32-bit
    // byte offset of the lane that only depends on sb (the wave's row block in the superblock, clamped to the
    // linear's last one for a wave that idles, and the lane's place in a tile): the instruction takes both as they
    // are, and the arithmetic per load stays on the scalar unit.
    struct LaneOffs {
        uint32_t w, s;       // into the codes; into scales / zeros (grouped scheme)
    };
    constexpr int LANE_BYTES = V == V_W3 ? 12 : 16, TILE = VInfo<V>::TILE_BYTES;
    // Wide path, 3/4-bit codes: a 32x32x16 B operand is tiles (p, p + 2) of the wave's block with lanes 0-15 / 16-31 on
    // the two tiles and lanes 32-63 two k slots further on.  A lane loads what it will hold -- the packed codes of lane
    // r + 32 * khalf (+ 16 for the second operand) of tile p + 2 * sel, r = lane % 16, sel = lane / 16 % 2, khalf =
    // lane / 32: the same bytes of the same tiles, in another lane order -- instead of every tile in its own order and
    // an exchange of half the registers between lanes after unpacking.  Stage::w[p] is then pair p's operand of k slots
    // (kq 0, kq 2), w[p + 2] that of (kq 1, kq 3); the lane's row of the block is 4 r + p + 2 sel.
    constexpr bool PAIRED_LOADS = WIDE && (V == V_W3 || V == V_W4);
    static_assert(!PAIRED_LOADS || RT == 4, "two pairs of tiles per wave");
    auto lane_offs = [&](int sb) {
        const int wv = max(0, min(wave, row_blocks - 1 - sb * WAVES));
        const uint32_t sel = (uint32_t)(lane >> 4) & 1u;
        const uint32_t in_tile = PAIRED_LOADS ? 2u * sel * TILE + LANE_BYTES * (uint32_t)(r + 32 * (lane >> 5)) : LANE_BYTES * (uint32_t)lane;
        LaneOffs o;
        if constexpr (RT == 4) o.w = (uint32_t)wv * (uint32_t)KT * (4u * TILE) + in_tile;
        else o.w = ((uint32_t)(wv >> 1) * (uint32_t)KT * 4u + 2u * (uint32_t)(wv & 1)) * TILE + in_tile;      // half a 64-row block per wave
        o.s = ((uint32_t)wv * 64u + 4u * (uint32_t)r + (PAIRED_LOADS ? 2u * sel : 0u)) * 2u;
        return o;
    };
    auto issue = [&](Stage& b, int sb, int kt, LaneOffs& o) {
        const uint8_t* wbase = L.codes + ((size_t)sb * (WAVES * RT / 4) * KT + kt) * (4 * (size_t)TILE);
        asm volatile("" : "+v"(o.w));        // widened next to the loads, so that base and offset stay apart
#pragma unroll
        for (int t = 0; t < RT; ++t) b.w[t] = load_tile_at<V>(wbase + o.w + (PAIRED_LOADS ? (t & 1) * TILE + (t >> 1) * 16 * LANE_BYTES : t * TILE));
        if constexpr (SCHEME == SCH_ASYM) {
            const size_t row0 = ((size_t)kt * L.N + (size_t)sb * (WAVES * 64)) * 2;
            asm volatile("" : "+v"(o.s));
            if constexpr (PAIRED_LOADS) {    // the lane's two rows: of pair 0 and of pair 1
                b.s[0] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(L.scales) + row0 + o.s);
                b.z[0] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(L.zeros) + row0 + o.s);
            } else {
                b.s = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(L.scales) + row0 + o.s);
                if constexpr (!POST) b.z = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(L.zeros) + row0 + o.s);
            }
        }
    };
    // Two ways to fold scale and zero in.  POST (up to 32 tokens): multiply raw codes (as fp16
    // subnormals, code * 2^-24) on the matrix cores per 128-column group, then acc += scale *
    // (codes . x) in fp32 -- unpacking a code is then a shift and a mask, and the fold costs 4 fp32
    // FMAs per tile and token tile instead of the int -> fp16 conversions and packed FMAs per weight.
    // The zero term, sum over groups of zero[n][g] * sum_g(x[m]), is itself a small matrix product
    // (K / 128 deep): it is added once per unit, at its end, from the group sums that
    // decode_prepare_kernel left in prep (add_zero_term below).  Otherwise (64 tokens, where the fp32
    // work has outgrown the saving): dequantise each weight to fp16 once, w~ = scale * code + zero.
    // MFMA A operand: 8 consecutive columns (16-byte group c16 of 128-column step `step`) of a token row
    auto x_operand = [&](int buf, int row, int step, int c16) {
        return *reinterpret_cast<const h8*>(&sm.x[buf][row][step * 128 + 8 * (c16 ^ (row & 15))]);
    };
    auto compute = [&](Stage& b, int buf, int step) {
        if constexpr (WIDE) {
            // dequantise two MFMA steps of every tile at a time, pair tiles (p, p + NP) into 32-row
            // operands (wb[p] then holds k slots kq 0 and 2, wb[p + NP] slots kq 1 and 3), multiply
            const int arow = lane & 31, ahalf = lane >> 5;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                h8 wb[RT][2];
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    unpack_codes_half<V>(b.w[t], half, wb[t]);
                    if constexpr (SCHEME == SCH_ASYM) {
                        const uint32_t sp = b.s[PAIRED_LOADS ? 0 : t >> 1], zp = b.z[PAIRED_LOADS ? 0 : t >> 1];      // PAIRED_LOADS: operand t belongs to pair t & 1
                        const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                        const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                        apply_scale_zero_half(wb[t], __builtin_bit_cast(_Float16, sh), __builtin_bit_cast(_Float16, zh));
                    }
                }
                if constexpr (!PAIRED_LOADS)
#pragma unroll
                    for (int p = 0; p < NP; ++p)
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) pair_tiles_for_mfma32(wb[p][jj], wb[p + NP][jj]);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int j = 2 * half + jj;
#pragma unroll
                    for (int m2 = 0; m2 < MT2; ++m2) {
                        const h8 a0 = x_operand(buf, 32 * m2 + arow, step, 4 * j + 2 * ahalf);
                        const h8 a1 = x_operand(buf, 32 * m2 + arow, step, 4 * j + 2 * ahalf + 1);
#pragma unroll
                        for (int p = 0; p < NP; ++p) {
                            accw[p][m2] = mfma32(a0, wb[p][jj], accw[p][m2]);
                            accw[p][m2] = mfma32(a1, wb[p + NP][jj], accw[p][m2]);
                        }
                    }
                }
            }
            return;
        }
        if constexpr (POST && !WIDE) {
            // In-order issue: vector work in front of a run of matrix instructions is not hidden by
            // them, vector work between them is.  So the codes of MFMA step j + 1 are unpacked in the
            // same scheduling group as the matrix instructions of step j.
            h8 wj[2][RT];
            const f4 zero4 = {0, 0, 0, 0};
            f4 d[RT][MT];
#pragma unroll
            for (int t = 0; t < RT; ++t) wj[0][t] = unpack_post<V, INPLACE>(b.w[t], 0);
            h8 a[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[0][mt] = x_operand(buf, 16 * mt + r, step, kq);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // one scheduling group per tile: its matrix instruction(s) of step j and the unpacking of the same
                // tile for step j + 1, so that the vector work sits between matrix instructions, not in front of them
                if (j < 3) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) a[(j + 1) & 1][mt] = x_operand(buf, 16 * mt + r, step, 4 * (j + 1) + kq);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    if (j < 3) wj[(j + 1) & 1][t] = unpack_post<V, INPLACE>(b.w[t], j + 1);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        if constexpr (SCHEME == SCH_ASYM) d[t][mt] = mfma16(a[j & 1][mt], wj[j & 1][t], j == 0 ? zero4 : d[t][mt]);
                        else                               acc[t][mt] = mfma16(a[j & 1][mt], wj[j & 1][t], acc[t][mt]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (SCHEME == SCH_ASYM) {
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    const float sf = (float)as_h2(b.s[t >> 1])[t & 1];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[t][mt][v] = __builtin_fmaf(sf, d[t][mt][v], acc[t][mt][v]);
                }
            }
        } else {
            h8 wb[RT][4];
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                unpack_codes<V>(b.w[t], wb[t]);
                if constexpr (SCHEME == SCH_ASYM) {
                    const uint32_t sp = b.s[t >> 1], zp = b.z[t >> 1];
                    const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                    const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                    apply_scale_zero(wb[t], __builtin_bit_cast(_Float16, sh), __builtin_bit_cast(_Float16, zh));
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const h8 a = x_operand(buf, 16 * mt + r, step, 4 * j + kq);
#pragma unroll
                    for (int t = 0; t < RT; ++t) acc[t][mt] = mfma16(a, wb[t][j], acc[t][mt]);
                }
        }
    };

    // INPLACE: rows 0 .. of this pass of the activations that decode_prepare_kernel scaled, behind the linear's 32 rows of group sums
    const uint16_t* xrows = INPLACE ? prep + (size_t)L.aux * 8 + (size_t)32 * group_sums_stride(L.K()) : L.x;
    const int xrow0 = INPLACE ? 0 : m0, xrow_last = INPLACE ? min(TOK, M - m0) - 1 : M - 1;
    // ---- activation staging: the x columns of one chunk, shared by the workgroup through LDS.
    // Global-to-LDS loads, 1 KB per wave and instruction (four 256-byte row segments); a lane fetches
    // the column group that belongs in its 16-byte slot after swizzling.  Token rows past M and steps
    // past the end of a short chunk are clamped to valid ones: they feed nothing that is stored.
    // The loads are asynchronous: wait on vmcnt before the barrier that publishes the buffer.
    auto fill_x_chunk = [&](const Chunk& c, int buf) {
#pragma unroll
        for (int i = 0; i < XQ; ++i) {
            const int q = XQ * wave + i;
            const int u = 4 * q + (lane >> 4), row = u / CHUNK, seg = min(u % CHUNK, c.n - 1);
            const int c16 = (lane & 15) ^ (row & 15);
            const uint16_t* g = xrows + (size_t)min(xrow0 + row, xrow_last) * L.K() + (size_t)(c.kt0 + seg) * 128 + c16 * 8;
            __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)(&sm.x[buf][0][0] + 512 * q), 16, 0, 0);
        }
        asm volatile("" ::: "memory");      // weight loads issued later stay later: vmcnt counts in issue order
    };

    // ---- end of a unit: lane holds tokens 4*kq + v of RT consecutive rows starting at nbase
    auto finish_unit = [&](int sb, float* __restrict__ partial) {
        const long rb = row_block(sb);
        if (WIDE && rb < row_blocks) {
            // lane (n = lane%32, half = lane/32) holds tokens 32*m2 + 8*(v/4) + 4*half + v%4 of NP consecutive rows:
            // tile pair p of a 4-tile block is tiles (p, p+2), i.e. rows 4r + p (n < 16) and 4r + 2 + p (n >= 16)
            const int ncol = lane & 31;
            int thalf = lane >> 5;
            // opaque to the optimiser: otherwise it precomputes every token's row offset (tok * N) ahead
            // of the main loop and keeps dozens of registers live across it for this rare path
            asm volatile("" : "+v"(thalf));
            const long nbase = (RT == 4) ? rb * 64 + 4 * (ncol & 15) + 2 * (ncol >> 4)
                                         : (rb >> 1) * 64 + 4 * (ncol & 15) + 2 * (rb & 1) + (ncol >> 4);
            float post[NP], bias[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                post[p] = 1.0f;
                if constexpr (SCHEME == SCH_SYM) post[p] = (float)__builtin_bit_cast(_Float16, L.scales[nbase + p]);
                bias[p] = (L.bias && !partial) ? (float)__builtin_bit_cast(_Float16, L.bias[nbase + p]) : 0.0f;
            }
#pragma unroll
            for (int m2 = 0; m2 < MT2; ++m2)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tok = m0 + 32 * m2 + 8 * (v / 4) + 4 * thalf + (v % 4);
                    if (tok >= M) continue;
                    if (!partial) {
                        typedef _Float16 hv __attribute__((ext_vector_type(NP)));
                        hv o, res;
                        if (L.residual) res = *reinterpret_cast<const hv*>(L.residual + (size_t)tok * L.N + nbase);
#pragma unroll
                        for (int p = 0; p < NP; ++p) {
                            float val = apply_activation(accw[p][m2][v] * post[p] + bias[p], L.act);
                            if (L.residual) val += (float)res[p];
                            o[p] = (_Float16)val;
                        }
                        *reinterpret_cast<hv*>(L.y + (size_t)tok * L.N + nbase) = o;
                    } else {
                        typedef float fv __attribute__((ext_vector_type(NP)));
                        fv o;
#pragma unroll
                        for (int p = 0; p < NP; ++p) o[p] = accw[p][m2][v] * post[p];
                        *reinterpret_cast<fv*>(partial + (size_t)(tok - m0) * (WAVES * 64) + (nbase - (long)sb * (WAVES * 16 * RT))) = o;
                    }
                }
        }
        if (!WIDE && rb < row_blocks) {
            const long nbase = (RT == 4) ? rb * 64 + 4 * r : (rb >> 1) * 64 + 4 * r + 2 * (rb & 1);
            if constexpr (POST) {
                // The accumulators hold y * 2^-24 without the zero term: the grouped scheme's sum over groups of
                // zero[n][g] * sum_g(x[m]), the per-row scheme's -128 * sum(x[m]) for the offset of its codes.  That
                // term is a matrix product over the groups this range covered, [tokens][groups] . [groups][rows], with
                // each group sum as an fp16 pair hi + lo in two adjacent k slots, scaled per token row (see
                // decode_prepare_kernel): bring the accumulators to y * scale, chain the product onto them, 16 groups
                // per matrix instruction, then divide the scale out.
                static_assert(RT == 4, "the zero term reads the zeros of a 64-row block");
                const long u0 = (long)sb * KT;
                const int g_lo = (int)(max(u0, s_begin) - u0), g_hi = (int)(min(u0 + KT, s_end) - u0);
                const int stride = group_sums_stride(L.K());
                const uint16_t* xs = prep + (size_t)L.aux * 8;
                const int cnt = min(TOK, M - m0);                            // token rows the sums were taken for
                float undo[MT][4];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float* f = reinterpret_cast<const float*>(xs + (size_t)min(16 * mt + 4 * kq + v, cnt - 1) * stride + (stride - 8));
                        const float pre = f[0];
                        undo[mt][v] = f[1];
#pragma unroll
                        for (int t = 0; t < RT; ++t) acc[t][mt][v] *= pre;
                    }
                // CB matrix steps (16 groups each) per round of loads: a round costs a memory latency that nothing hides
                constexpr int CB = TOK <= 16 ? 4 : 1;
                const int c_last = (KT + 15) / 16 - 1;                       // the sums are padded to whole matrix steps
                for (int c0 = g_lo >> 4; 16 * c0 < g_hi; c0 += CB) {
                    h8 a[CB][MT];
                    u32x2 z[CB][4];
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        const int c = min(c0 + cb, c_last);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            a[cb][mt] = *reinterpret_cast<const h8*>(xs + (size_t)min(16 * mt + r, cnt - 1) * stride + 32 * c + 8 * kq);
                        if constexpr (SCHEME == SCH_ASYM) {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                z[cb][i] = *reinterpret_cast<const u32x2*>(L.zeros + (size_t)min(16 * c + 4 * kq + i, KT - 1) * L.N + rb * 64 + 4 * r);
                        }
                    }
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        u32x4 bz[RT];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int g = 16 * (c0 + cb) + 4 * kq + i;       // k slots 8 kq + 2 i and + 1
                            const bool valid = g >= g_lo && g < g_hi;
#pragma unroll
                            for (int t = 0; t < RT; ++t) {
                                uint32_t h = 0xd800u;                        // per-row scheme: -128
                                if constexpr (SCHEME == SCH_ASYM) h = (t & 1) ? (z[cb][i][t >> 1] >> 16) : (z[cb][i][t >> 1] & 0xffffu);
                                bz[t][i] = valid ? (h | (h << 16)) : 0u;
                            }
                        }
#pragma unroll
                        for (int t = 0; t < RT; ++t)
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt) acc[t][mt] = mfma16(a[cb][mt], __builtin_bit_cast(h8, bz[t]), acc[t][mt]);
                    }
                }
#pragma unroll
                for (int t = 0; t < RT; ++t)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[t][mt][v] *= undo[mt][v];
            }
            float post[RT], bias[RT];
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                post[t] = 1.0f;
                if constexpr (SCHEME == SCH_SYM) post[t] = (float)__builtin_bit_cast(_Float16, L.scales[nbase + t]);
                bias[t] = (L.bias && !partial) ? (float)__builtin_bit_cast(_Float16, L.bias[nbase + t]) : 0.0f;
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int tok = m0 + 16 * mt + 4 * kq + v;
                    if (tok >= M) continue;
                    float val[RT];
#pragma unroll
                    for (int t = 0; t < RT; ++t) {
                        val[t] = acc[t][mt][v] * post[t];
                    }
                    if (!partial) {
                        typedef _Float16 hv __attribute__((ext_vector_type(RT)));
                        hv o, res;
                        if (L.residual) res = *reinterpret_cast<const hv*>(L.residual + (size_t)tok * L.N + nbase);
#pragma unroll
                        for (int t = 0; t < RT; ++t) {
                            float e = apply_activation(val[t] + bias[t], L.act);
                            if (L.residual) e += (float)res[t];
                            o[t] = (_Float16)e;
                        }
                        *reinterpret_cast<hv*>(L.y + (size_t)tok * L.N + nbase) = o;
                    } else {
                        typedef float fv __attribute__((ext_vector_type(RT)));
                        fv o;
#pragma unroll
                        for (int t = 0; t < RT; ++t) o[t] = val[t];
                        *reinterpret_cast<fv*>(partial + (size_t)(tok - m0) * (WAVES * 64) + (nbase - (long)sb * (WAVES * 16 * RT))) = o;
                    }
                }
        }
        clear_acc();
    };

    // ---- main loop over chunks; loads for slot i + STAGES are issued right after slot i is consumed,
    // whether that slot lies in this chunk or in the next one (possibly of the next unit)
    Chunk cur = first_chunk(s_begin), nxt = next_chunk(cur);
    LaneOffs oc = lane_offs(cur.sb), on = lane_offs(nxt.sb);
    fill_x_chunk(cur, 0);
#pragma unroll
    for (int i = 0; i < STAGES; ++i)
        if (i < cur.n) issue(st[i], cur.sb, cur.kt0 + i, oc);      // slots past a short chunk stay empty
    wait_vmem_all_but<0>();
    __syncthreads();
    int buf = 0;
    while (cur.n > 0) {
        if (nxt.n > 0) fill_x_chunk(nxt, buf ^ 1);
        const bool active = row_block(cur.sb) < row_blocks;
        // steady state: a chunk of N steps (a full one; in the 16-step form also a linear's remainder of exactly 8)
        // followed by enough steps to refill every slot -- no per-step conditions, so the whole chunk is one
        // schedulable block
        auto steady_chunk = [&](auto n_steps) {
            constexpr int N = decltype(n_steps)::value;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                compute(st[i % STAGES], buf, i);
                const int q = i + STAGES;                   // slot to refill
                if (q < N) issue(st[i % STAGES], cur.sb, cur.kt0 + q, oc);
                else       issue(st[i % STAGES], nxt.sb, nxt.kt0 + (q - N), on);
                if constexpr (WIDE) __builtin_amdgcn_sched_barrier(0);      // keeps a step's operand reads out of earlier steps (register pressure)
            }
            // the next chunk's activations were requested before this chunk's last STAGES refills, which stay in flight
            wait_vmem_all_but<STAGES * STAGE_LOADS>();
        };
        if (cur.n == CHUNK && active && nxt.n >= STAGES) {
            steady_chunk(std::integral_constant<int, CHUNK>());
        } else if (CHUNK == 16 && cur.n == 8 && active && nxt.n >= STAGES) {
            steady_chunk(std::integral_constant<int, CHUNK == 16 ? 8 : CHUNK>());
        } else {
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) {
                if (i < cur.n && active) compute(st[i % STAGES], buf, i);
                const int q = i + STAGES;
                if (q < CHUNK) { if (q < cur.n) issue(st[i % STAGES], cur.sb, cur.kt0 + q, oc); }
                else           { if (q - CHUNK < nxt.n) issue(st[i % STAGES], nxt.sb, nxt.kt0 + (q - CHUNK), on); }
            }
            wait_vmem_all_but<0>();
        }
        const bool unit_ends = cur.kt0 + cur.n == KT || nxt.n == 0;
        if (unit_ends) {
            const long u0 = (long)cur.sb * KT;               // the unit's first step
            const bool whole = u0 >= s_begin && u0 + KT <= s_end;
            finish_unit(cur.sb, whole ? nullptr : (u0 < s_begin ? slot_first : slot_last));
        }
        __syncthreads();
        buf ^= 1;
        cur = nxt;
        nxt = next_chunk(nxt);
        oc = on;
        if (nxt.sb != cur.sb) on = lane_offs(nxt.sb);
    }
}

// Position of a workgroup's range in the weighted step list.
struct Cursor {
    int li;          // linear
    long step;       // block step inside the linear: sb * KT + kt
};

// floor(n / d) for n < 2^52 through one double-precision division: the quotient's integer part is off by at most
// one, which the product shows.  (The 64-bit integer division it replaces is some two hundred instructions, and the
// kernels here do several in a row before their first load.)
__device__ __forceinline__ uint64_t div_floor(uint64_t n, uint32_t d)
{
    uint64_t q = (uint64_t)((double)n / (double)d);
    const uint64_t p = q * d;
    if (p > n) --q;
    else if (n - p >= d) ++q;
    return q;
}

// first step whose start offset is >= pos (pos <= total weight)
__device__ __forceinline__ Cursor first_step_at(const DecodeArgs& a, uint64_t pos)
{
    int li = 0, hi = a.n_lin - 1;                    // last linear whose cum_weight <= pos
    while (li < hi) {
        const int mid = (li + hi + 1) >> 1;
        if (a.lin[mid].cum_weight <= pos) li = mid; else hi = mid - 1;
    }
    const LinDesc& L = a.lin[li];
    const uint64_t off = pos - L.cum_weight;
    Cursor c = {li, (long)div_floor(off + L.step_weight - 1, L.step_weight)};
    return c;
}

__device__ __forceinline__ uint64_t range_begin(const DecodeArgs& a, int b)
{
    // floor(total_weight * b / n_blocks), total_weight < 2^50, b <= n_blocks < 2^13: the remainder's share needs 32 bits only
    return a.range_q * (uint64_t)b + (a.range_rem * (uint32_t)b) / (uint32_t)a.n_blocks;
}

// What a decode launch of up to 32 token rows per pass needs from its activations beforehand.  Workgroup
// (blockIdx.x = linear, blockIdx.y = row of the pass) reads token row a.m0 + row of the linear's x once and writes, at
// prep + 8 * aux halves:
//  - the group sums for the zero term: x added over each 128-column group (sixteen lanes per group, a fixed order), as
//    fp16 pairs for the matrix cores: sum * scale = hi + lo (lo = the rounding error of hi), scale the power of two that
//    brings the row's largest |sum| into [2^13, 2^14) -- so that rows of tiny activations keep their bits and rows of
//    large ones stay in range.  A row is group_sums_stride(K) halves: the pairs of groups 0 .. K/128 - 1, zero pairs up
//    to a multiple of 16 groups (they meet zero operands, but must not be NaN), then two floats, pre and undo: the
//    accumulators are multiplied by pre before the zero term is chained onto them and by undo afterwards;
//  - for 3-bit weights that the launch reads in place (variant V_W3_INPLACE), behind the 32 rows of sums: the row scaled for codes that are masked where they lie
//    (unpack_inplace_step): column c of a 128-column step times 2^-(3 * inplace_class(c / 32, (c % 8) / 2)), times the
//    power of two that brings the row's largest |x| into [2^14, 2^15) -- exact, and with the row at the
//    top of the fp16 range the factors of up to 2^-6 cost only elements 2^23 below the row's largest any bits.  pre
//    carries the inverse of that power.
// The kernel is a round of memory latency in front of every decode launch, so a workgroup is 1024 threads (64 groups at a
// time) and a thread requests all it adds -- up to GS_ROUNDS groups, K <= 65536 -- before it adds anything, keeping
// the sums in registers for the second use; a longer row is read twice.
constexpr int GS_THREADS = 1024, GS_ROUNDS = 8, GS_LANES = 16, GS_GROUPS = GS_THREADS / GS_LANES;

template <bool ANY_INPLACE>
__global__ __launch_bounds__(GS_THREADS) void decode_prepare_kernel(const DecodeArgs a, uint16_t* __restrict__ prep)
{
    __shared__ float wmax[2][GS_THREADS / 64];
    const LinDesc& L = a.lin[blockIdx.x];
    if (L.variant == V_F16) return;
    const bool scaled = ANY_INPLACE && L.variant == V_W3_INPLACE;
    constexpr int width = 3;
    const int row = blockIdx.y, tok = a.m0 + row;
    const int KT = L.K() / 128, GP = (KT + 15) & ~15, rounds = (GP + GS_GROUPS - 1) / GS_GROUPS;
    uint16_t* base = prep + (size_t)L.aux * 8;
    uint16_t* dst = base + (size_t)row * group_sums_stride(L.K());
    uint16_t* xq = base + (size_t)32 * group_sums_stride(L.K()) + (size_t)row * L.K();
    const int l16 = threadIdx.x & 15, g0 = threadIdx.x >> 4;
    const uint16_t* src = L.x + (size_t)tok * L.K() + 8 * l16;
    auto load = [&](int g) { return *reinterpret_cast<const h8*>(src + (size_t)min(g, KT - 1) * 128); };
    auto add16 = [&](h8 v, bool valid) {              // a group's sum, the same value in all sixteen lanes
        float sum = (((float)v[0] + (float)v[1]) + ((float)v[2] + (float)v[3])) + (((float)v[4] + (float)v[5]) + ((float)v[6] + (float)v[7]));
        sum = valid ? sum : 0.0f;
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) sum += __shfl_xor(sum, o, 16);
        return sum;
    };
    auto largest = [&](h8 v) {
        float m = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf((float)v[i]));
        return m;
    };
    const bool fits = rounds <= GS_ROUNDS;
    h8 v[GS_ROUNDS];
    float sums[GS_ROUNDS];
    float big = 0.0f, xbig = 0.0f;
    if (fits) {
#pragma unroll
        for (int i = 0; i < GS_ROUNDS; ++i)
            if (i < rounds) v[i] = load(g0 + GS_GROUPS * i);                       // wave-uniform condition
#pragma unroll
        for (int i = 0; i < GS_ROUNDS; ++i) {
            sums[i] = i < rounds ? add16(v[i], g0 + GS_GROUPS * i < KT) : 0.0f;
            big = fmaxf(big, fabsf(sums[i]));
            if (scaled && i < rounds) xbig = fmaxf(xbig, largest(v[i]));           // a clamped group repeats a real one
        }
    } else {
        for (int g = g0; g < GP; g += GS_GROUPS) {
            const h8 u = load(g);
            big = fmaxf(big, fabsf(add16(u, g < KT)));
            if (scaled) xbig = fmaxf(xbig, largest(u));
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        big = fmaxf(big, __shfl_xor(big, o, 64));
        xbig = fmaxf(xbig, __shfl_xor(xbig, o, 64));
    }
    if ((threadIdx.x & 63) == 0) { wmax[0][threadIdx.x >> 6] = big; wmax[1][threadIdx.x >> 6] = xbig; }
    __syncthreads();
    big = xbig = 0.0f;
#pragma unroll
    for (int w = 0; w < GS_THREADS / 64; ++w) { big = fmaxf(big, wmax[0][w]); xbig = fmaxf(xbig, wmax[1][w]); }
    // the power of two that brings m into [2^(top-1), 2^top); 1 for a row of zeros (or one that holds an infinity)
    auto power_for = [](float m, int top) {
        if (!(m > 0.0f && m < __builtin_inff())) return 1.0f;
        int ex;
        (void)frexpf(m, &ex);                         // m = f * 2^ex, f in [0.5, 1)
        return ldexpf(1.0f, max(-40, min(40, top - ex)));
    };
    const float scale = power_for(big, 14);
    const float xscale = scaled ? power_for(xbig, 15) : 1.0f;
    auto store_sum = [&](int g, float sum) {
        const float sc = sum * scale;
        const _Float16 hi = (_Float16)sc;
        const _Float16 lo = (_Float16)(sc - (float)hi);
        if (l16 == 0 && g < GP)
            reinterpret_cast<uint32_t*>(dst)[g] = (uint32_t)__builtin_bit_cast(uint16_t, hi) | ((uint32_t)__builtin_bit_cast(uint16_t, lo) << 16);
    };
    // the lane's eight columns are columns 8 * (l16 % 4) .. + 7 of MFMA step l16 / 4: output registers k = 0 .. 3 of that step
    float mult[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        mult[k] = ldexpf(xscale, -width * inplace_class<V_W3>(l16 >> 2, k));
    }
    auto store_row = [&](int g, h8 u) {
        if (g >= KT) return;
        h8 o;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = (_Float16)((float)u[i] * mult[i >> 1]);
        *reinterpret_cast<h8*>(xq + (size_t)g * 128 + 8 * l16) = o;
    };
    if (fits) {
#pragma unroll
        for (int i = 0; i < GS_ROUNDS; ++i)
            if (i < rounds) store_sum(g0 + GS_GROUPS * i, sums[i]);
        // the row is read once more (from the caches) rather than kept: the registers would halve the workgroups a CU holds
        if (scaled)
            for (int g = g0; g < KT; g += GS_GROUPS) store_row(g, load(g));
    } else {
        for (int g = g0; g < GP; g += GS_GROUPS) {
            const h8 u = load(g);
            store_sum(g, add16(u, g < KT));
            if (scaled) store_row(g, u);
        }
    }
    if (threadIdx.x == 0) {
        float* f = reinterpret_cast<float*>(dst + 2 * GP);
        f[0] = scale * 16777216.0f / xscale;
        f[1] = 1.0f / scale;
    }
}

template <int TOK, int WAVES, int CAP>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void decode_kernel(const DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    DecodeSmem<TOK, WAVES, CAP>& sm = *reinterpret_cast<DecodeSmem<TOK, WAVES, CAP>*>(smem_raw);
    // Workgroup ids go round-robin over the 8 XCDs, each with its own L2.  XCD x takes the x-th eighth of the
    // ranges, so that a linear's activations are fetched into one or two L2s instead of all eight.
    const int b = (a.n_blocks & 7) == 0 ? (int)(blockIdx.x & 7) * (a.n_blocks >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const uint64_t lo = range_begin(a, b), hi = range_begin(a, b + 1);
    Cursor c = first_step_at(a, lo);
    float* slot_first = a.partial + (size_t)(2 * b) * a.slot_floats;
    float* slot_last = slot_first + a.slot_floats;
    while (c.li < a.n_lin) {
        const LinDesc& L = a.lin[c.li];
        const long steps = (long)lin_row_superblocks(L, WAVES) * L.kt;
        if (c.step >= steps) { ++c.li; c.step = 0; continue; }
        const uint64_t start = L.cum_weight + (uint64_t)c.step * L.step_weight;
        if (start >= hi) break;
        const long budget = (long)((hi - start + L.step_weight - 1) / L.step_weight);      // steps of this range from here
        const long s_end = min(steps, c.step + budget);
        switch (L.variant) {
        case V_W3: run_range<V_W3, TOK, WAVES, CAP>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm); break;
        case V_W3_INPLACE:
            if constexpr (TOK <= 16) run_range<V_W3, TOK, WAVES, CAP, true>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm);
            break;
        case V_W4: run_range<V_W4, TOK, WAVES, CAP>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm); break;
        case V_W8: run_range<V_W8, TOK, WAVES, CAP>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm); break;
        case V_I8: run_range<V_I8, TOK, WAVES, CAP>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm); break;
        default:   run_range<V_F16, TOK, WAVES, CAP>(L, a.M, a.m0, c.step, s_end, a.prep, slot_first, slot_last, sm); break;
        }
        c.step = s_end;
    }
}

// Fix-up: workgroup b looks at the boundary between ranges b and b+1.  If it is the first boundary
// that cuts a unit, this workgroup adds that unit's pieces (range b's last segment, then the first
// segments of ranges b+1, b+2, ... until the unit ends), adds the bias and stores fp16.
__global__ __launch_bounds__(256) void decode_fixup_kernel(const DecodeArgs a)
{
    const int b = blockIdx.x;                       // 0 .. n_blocks - 2
    const uint64_t X = range_begin(a, b + 1);
    const Cursor c = first_step_at(a, X);
    const LinDesc& L = a.lin[c.li];
    const int KT = L.kt;
    const long steps = (long)lin_row_superblocks(L, 8) * KT;       // this kernel follows the eight-wave launches only
    if (c.step >= steps || c.step % KT == 0) return;            // boundary falls between units
    const int sb = (int)(c.step / KT);
    const uint64_t unit_begin = L.cum_weight + (uint64_t)sb * KT * L.step_weight;
    if (range_begin(a, b) > unit_begin) return;                 // an earlier boundary already cuts this unit
    const uint64_t unit_end = unit_begin + (uint64_t)KT * L.step_weight;     // start offset of the next unit
    // pieces: slot 2b+1, then slot 2b' for every later non-empty range b' whose first step lies in this unit
    const int rows_wg = a.waves * decode_rows_per_wave(L.variant);      // rows of W per workgroup in this linear
    const int stride = a.waves * 64;                                    // floats per token row of a partial tile
    const long nbase = (long)sb * rows_wg;
    const int m_cnt = min(64, a.M - a.m0);
    // A pass covers 1024 groups of 4 consecutive rows (16 tokens of a four-wave workgroup's rows).  Every
    // piece costs a round of memory latency, so a unit cut into many pieces (a single small linear spread
    // over the whole chip) has them dealt round-robin to the four waves, each wave adding its pieces for
    // all 1024 groups, and the four sums are then added in a fixed order through LDS; a unit cut into a few
    // pieces (the usual case in a stage-wide launch) is added by all threads piece after piece.
    // Deterministic either way.
    constexpr int PER_LANE = 16, PER_THREAD = 4;
    __shared__ f4 wsum[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_items = m_cnt * (rows_wg / 4);
    auto for_each_piece = [&](auto&& fn) {         // slot 2b+1, then slot 2b' of every later non-empty range that starts in this unit
        fn(2 * b + 1);
        uint64_t lo = X;
        for (int bb = b + 1; bb < a.n_blocks; ++bb) {
            const uint64_t next = range_begin(a, bb + 1);
            const uint64_t first = L.cum_weight + div_floor(lo - L.cum_weight + L.step_weight - 1, L.step_weight) * L.step_weight;
            if (first >= unit_end) break;
            if (first < next) fn(2 * bb);                       // else an empty range: it wrote nothing
            lo = next;
        }
    };
    // bias and residual of an item do not depend on the pieces: they are requested ahead of them, so that their
    // round of memory latency runs beside the pieces' instead of behind it
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    struct Extra { h4 bias, res; };
    auto fetch = [&](int idx) {
        Extra e = {h4{0, 0, 0, 0}, h4{0, 0, 0, 0}};
        if (idx >= n_items) return e;
        const int tok = idx / (rows_wg / 4), n4 = (idx % (rows_wg / 4)) * 4;
        if (nbase + n4 >= L.N) return e;
        if (L.bias) e.bias = *reinterpret_cast<const h4*>(L.bias + nbase + n4);
        if (L.residual) e.res = *reinterpret_cast<const h4*>(L.residual + (size_t)(a.m0 + tok) * L.N + nbase + n4);
        return e;
    };
    auto finish = [&](int idx, f4 sv, const Extra& e) {            // bias, activation, residual, one rounding
        if (idx >= n_items) return;
        const int tok = idx / (rows_wg / 4), n4 = (idx % (rows_wg / 4)) * 4;
        if (nbase + n4 >= L.N) return;
        if (L.bias)
#pragma unroll
            for (int v = 0; v < 4; ++v) sv[v] += (float)e.bias[v];
#pragma unroll
        for (int v = 0; v < 4; ++v) sv[v] = apply_activation(sv[v], L.act);
        if (L.residual)
#pragma unroll
            for (int v = 0; v < 4; ++v) sv[v] += (float)e.res[v];
        const h4 out = {(_Float16)sv[0], (_Float16)sv[1], (_Float16)sv[2], (_Float16)sv[3]};
        *reinterpret_cast<h4*>(L.y + (size_t)(a.m0 + tok) * L.N + nbase + n4) = out;
    };
    // ranges that overlap the unit (an upper bound that needs no walk): unit weight / range weight, plus both ends
    const uint64_t n_pieces = (uint64_t)((double)((uint64_t)KT * L.step_weight) / (double)max(a.range_q, (uint64_t)1)) + 2;
    // blockIdx.y picks the pass: a unit of 64 tokens x 512 rows is eight passes, added by eight workgroups
    const int base = (int)blockIdx.y * 1024;
    if (base < n_items) {
        if (n_pieces <= 4) {
            f4 sum[PER_THREAD];
            size_t off[PER_THREAD];
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const int idx = base + threadIdx.x + 256 * i;
                off[i] = (size_t)(idx / (rows_wg / 4)) * stride + (idx % (rows_wg / 4)) * 4;
                sum[i] = f4{0, 0, 0, 0};
            }
            Extra extra[PER_THREAD];
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) extra[i] = fetch(base + threadIdx.x + 256 * i);
            for_each_piece([&](int slot) {         // all of a piece's loads are issued before the first add
                const float* p = a.partial + (size_t)slot * a.slot_floats;
                f4 v[PER_THREAD];
#pragma unroll
                for (int i = 0; i < PER_THREAD; ++i)
                    if (base + threadIdx.x + 256 * i < n_items) v[i] = *reinterpret_cast<const f4*>(p + off[i]);
#pragma unroll
                for (int i = 0; i < PER_THREAD; ++i)
                    if (base + threadIdx.x + 256 * i < n_items) sum[i] += v[i];
            });
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) finish(base + threadIdx.x + 256 * i, sum[i], extra[i]);
            return;
        }
        f4 sum[PER_LANE];
        size_t off[PER_LANE];
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) {
            const int idx = base + lane + 64 * i;
            off[i] = (size_t)(idx / (rows_wg / 4)) * stride + (idx % (rows_wg / 4)) * 4;
            sum[i] = f4{0, 0, 0, 0};
        }
        int piece = 0;
        for_each_piece([&](int slot) {
            if ((piece++ & 3) != wave) return;
            const float* p = a.partial + (size_t)slot * a.slot_floats;
            f4 v[PER_LANE];
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i)
                if (base + lane + 64 * i < n_items) v[i] = *reinterpret_cast<const f4*>(p + off[i]);
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i)
                if (base + lane + 64 * i < n_items) sum[i] += v[i];
        });
#pragma unroll
        for (int q = 0; q < PER_LANE / 4; ++q) {                // groups base + 256q .. + 255
            __syncthreads();                                    // the previous round has read wsum
#pragma unroll
            for (int i = 0; i < 4; ++i) wsum[wave][lane + 64 * i] = sum[4 * q + i];
            __syncthreads();
            finish(base + 256 * q + threadIdx.x,
                   (wsum[0][threadIdx.x] + wsum[1][threadIdx.x]) + (wsum[2][threadIdx.x] + wsum[3][threadIdx.x]),
                   fetch(base + 256 * q + threadIdx.x));
        }
    }
}

// ---- small launches (one linear of a decoder layer, up to 32 token rows = MT token tiles of 16) ---------------
// The even-share kernel above needs a launch with many steps to spread; a single linear has few, and cutting
// its units into short ranges leaves each workgroup waiting on memory latency and pays a fix-up pass.  Here a
// workgroup owns a group of TILES consecutive 16-row tiles of W (at most 2 for fp16 weights) over the whole of
// K, and its waves split K: wave w takes the 128-column steps w, w + WAVES, ...  Four tiles are one 64-row
// block of the packed layout; groups of 3 or 5 tiles cut across blocks, so that the host can pick the group
// size whose workgroups just fill the compute units once (1280 tiles = 256 groups of 5).  Each wave streams its
// tiles through a ring of stages in registers together with the activations of those steps (read straight from
// global memory: they are small and stay in L2; no LDS staging, no barrier in the loop), and the waves'
// accumulators are added through LDS at the end, in wave order.  A linear with few tiles and a long K (the
// second feed-forward matrix) is also split over L.aux workgroups per group, each taking a range of the steps
// and leaving fp32 sums in partial[split][16 MT][N] (at float offset L.step_weight of the launch's partial buffer)
// for a small second kernel; otherwise there are no partial tiles and no second kernel.  rows_row_blocks(L, row_tiles) is the
// linear's number of groups, a.lin[i].cum_weight the number of workgroups of the linears before i, a.n_blocks
// their total.
template <int V, int WAVES, int TILES, int MT>
__device__ __forceinline__ void run_rows(const LinDesc& L, int M, long rb, int split, float* __restrict__ partial, float* __restrict__ red)
{
    constexpr int RT = (V == V_F16 && TILES > 2) ? 2 : TILES;      // 16-row tiles per workgroup; rb counts groups of RT tiles
    constexpr bool ALIGNED = RT == 2 || RT == 4;                    // the group lies in one 64-row block
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr bool POST = V != V_F16;
    constexpr int STAGES = (V == V_W3 || V == V_W4) ? 4 : 3;
    constexpr int LOADS = RT * (VInfo<V>::TILE_BYTES >= 1024 ? VInfo<V>::TILE_BYTES / 1024 : 1) +
                          (SCHEME == SCH_ASYM ? (ALIGNED ? 2 : 4) : 0) + 4 * MT;
    static_assert((STAGES - 1) * LOADS < 64, "vmcnt is a 6-bit counter");
    constexpr int NV = (RT * MT + (SCHEME == SCH_SYM ? MT : 0)) * 4;   // floats a lane hands to the reduction
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // a scalar: the row block and the tile addresses derive from it
    const int r = lane & 15, kq = lane >> 4;
    const int KT = L.K() / 128;
    const long g0 = rb * RT;                                        // first tile; tile g is tile g % 4 of 64-row block g / 4
    // the workgroup's steps [kt0, kt1): all of them, or the split's share (the first KT % splits take one more)
    const int splits = L.aux, share = KT / splits, extra = KT % splits;
    const int kt0 = split * share + min(split, extra), kt1 = kt0 + share + (split < extra ? 1 : 0);
    const int n_w = kt1 - kt0 > wave ? (kt1 - kt0 - wave + WAVES - 1) / WAVES : 0;      // this wave's steps
    const uint16_t* __restrict__ xrow[MT];                          // token tile m holds rows 16 m .. 16 m + 15; rows past M repeat the last one
#pragma unroll
    for (int m = 0; m < MT; ++m) xrow[m] = L.x + (size_t)min(r + 16 * m, M - 1) * L.K() + 8 * kq;

    struct Stage {
        WRaw<V> w[RT];
        u32x2 s, z;                 // scales and zeros of rows 4 r .. 4 r + 3 of the first tile's block
        u32x2 s1, z1;               // !ALIGNED: and of the next block (the group spans two)
        h8 a[MT][4];
    };
    Stage st[STAGES];
    // step i of this wave; past its last step the loads repeat a valid step (they keep the count of loads in
    // flight constant, which is what the waits below rely on) and what they bring is never multiplied
    auto issue = [&](Stage& b, int i) {
        const int kt = min(kt0 + wave + WAVES * i, KT - 1);
#pragma unroll
        for (int t = 0; t < RT; ++t) b.w[t] = load_tile<V>(L.codes, (g0 + t) >> 2, KT, kt, (int)((g0 + t) & 3), lane);
        if constexpr (SCHEME == SCH_ASYM) {
            const size_t idx = (size_t)kt * L.N + (g0 >> 2) * 64 + 4 * r;
            b.s = *reinterpret_cast<const u32x2*>(L.scales + idx);
            b.z = *reinterpret_cast<const u32x2*>(L.zeros + idx);
            if constexpr (!ALIGNED) {
                const size_t idx1 = (size_t)kt * L.N + ((g0 + RT - 1) >> 2) * 64 + 4 * r;    // the last tile's block
                b.s1 = *reinterpret_cast<const u32x2*>(L.scales + idx1);
                b.z1 = *reinterpret_cast<const u32x2*>(L.zeros + idx1);
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) b.a[m][j] = *reinterpret_cast<const h8*>(xrow[m] + (size_t)kt * 128 + 32 * j);
    };

    f4 acc[RT][MT], xsum[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        xsum[m] = f4{0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < RT; ++t) acc[t][m] = f4{0, 0, 0, 0};
    }
    auto compute = [&](const Stage& b) {
        if constexpr (POST) {
            h8 wj[2][RT];
            const _Float16 one = (_Float16)1.0f;
            const h8 ones = {one, one, one, one, one, one, one, one};
            const f4 zero4 = {0, 0, 0, 0};
            f4 d[RT][MT], xs[MT];
#pragma unroll
            for (int t = 0; t < RT; ++t) wj[0][t] = unpack_subnormal_step<V>(b.w[t], 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // one scheduling group per tile: its matrix instructions of step j and the unpacking of the same tile
                // for step j + 1, so that the vector work sits between matrix instructions, not in front of them
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    if constexpr (SCHEME == SCH_ASYM) xs[m] = mfma16(b.a[m][j], ones, j == 0 ? zero4 : xs[m]);
                    else                               xsum[m] = mfma16(b.a[m][j], ones, xsum[m]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    if (j < 3) wj[(j + 1) & 1][t] = unpack_subnormal_step<V>(b.w[t], j + 1);
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        if constexpr (SCHEME == SCH_ASYM) d[t][m] = mfma16(b.a[m][j], wj[j & 1][t], j == 0 ? zero4 : d[t][m]);
                        else                               acc[t][m] = mfma16(b.a[m][j], wj[j & 1][t], acc[t][m]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (SCHEME == SCH_ASYM) {
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    const int tt = (int)((g0 + t) & 3);             // the tile's place in its block: row 4 r + tt
                    u32x2 s2 = b.s, z2 = b.z;
                    if constexpr (!ALIGNED) {
                        if (((g0 + t) >> 2) != (g0 >> 2)) s2 = b.s1, z2 = b.z1;     // uniform over the wave
                    }
                    const uint32_t sp = (tt >> 1) ? s2[1] : s2[0], zp = (tt >> 1) ? z2[1] : z2[0];
                    const uint16_t sh = (uint16_t)((tt & 1) ? (sp >> 16) : (sp & 0xffffu));
                    const uint16_t zh = (uint16_t)((tt & 1) ? (zp >> 16) : (zp & 0xffffu));
                    const float sf = (float)__builtin_bit_cast(_Float16, sh) * 16777216.0f;     // scale * 2^24
                    const float zf = (float)__builtin_bit_cast(_Float16, zh);
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[t][m][v] = __builtin_fmaf(sf, d[t][m][v], __builtin_fmaf(zf, xs[m][v], acc[t][m][v]));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int t = 0; t < RT; ++t)
#pragma unroll
                    for (int m = 0; m < MT; ++m) acc[t][m] = mfma16(b.a[m][j], __builtin_bit_cast(h8, b.w[t].q[j]), acc[t][m]);
        }
    };

#pragma unroll
    for (int sidx = 0; sidx < STAGES; ++sidx) issue(st[sidx], sidx);
    for (int i0 = 0; i0 < n_w; i0 += STAGES) {
#pragma unroll
        for (int sidx = 0; sidx < STAGES; ++sidx) {
            const int i = i0 + sidx;
            if (i < n_w) {                                        // uniform over the wave
                wait_vmem_all_but<(STAGES - 1) * LOADS>();       // stages i + 1 .. i + STAGES - 1 may still be in flight
                compute(st[sidx]);
                issue(st[sidx], i + STAGES);
            }
        }
    }

    // add the waves' sums in wave order; thread idx -> (token, row of the group), consecutive threads on consecutive rows
    float* mine = red + (size_t)wave * NV * 64;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[(4 * (t * MT + m) + v) * 64 + lane] = acc[t][m][v];
    if constexpr (SCHEME == SCH_SYM) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[(4 * (RT * MT + m) + v) * 64 + lane] = xsum[m][v];
    }
    __syncthreads();
    constexpr int ROWS = 16 * RT;
    for (int idx = tid; idx < 16 * MT * ROWS; idx += 64 * WAVES) {
        const int tok = idx / ROWS, rl = idx % ROWS;
        if (tok >= M) continue;
        const int m = tok >> 4, tl = tok & 15;
        const int rr = rl / RT, t = rl % RT, v = tl & 3, ln = 16 * (tl >> 2) + rr;
        float sum = 0.0f, xs = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[((size_t)w * NV + 4 * (t * MT + m) + v) * 64 + ln];
        const long row = ((g0 + t) >> 2) * 64 + 4 * rr + ((g0 + t) & 3);
        if constexpr (SCHEME == SCH_SYM) {
#pragma unroll
            for (int w = 0; w < WAVES; ++w) xs += red[((size_t)w * NV + 4 * (RT * MT + m) + v) * 64 + ln];
            sum = (sum * 16777216.0f - 128.0f * xs) * (float)__builtin_bit_cast(_Float16, L.scales[row]);   // undo 2^-24 and the +128 offset
        }
        const size_t o = (size_t)tok * L.N + row;
        if (splits > 1) {
            partial[((size_t)split * 16 * MT) * L.N + o] = sum;
            continue;
        }
        if (L.bias) sum += (float)__builtin_bit_cast(_Float16, L.bias[row]);
        sum = apply_activation(sum, L.act);
        if (L.residual) sum += (float)__builtin_bit_cast(_Float16, L.residual[o]);
        L.y[o] = __builtin_bit_cast(uint16_t, (_Float16)sum);
    }
}

// One token tile (up to 16 token rows): two workgroups of four waves per compute unit.  Two token tiles (17-32
// rows) double the activations of a stage, and five tiles of W fill the 256 registers of that occupancy: those
// kernels take up to 512 registers per lane and one four-wave workgroup per unit.
template <int WAVES, int TILES, int MT>
__global__ __launch_bounds__(64 * WAVES, (MT == 2 || TILES == 5) ? 1 : 8 / WAVES) void decode_rows_kernel(const DecodeArgs a)
{
    __shared__ float red[WAVES * (TILES * MT + MT) * 4 * 64];
    const int b = blockIdx.x;
    int li = 0, hi = a.n_lin - 1;                    // last linear whose first workgroup is <= b
    while (li < hi) {
        const int mid = (li + hi + 1) >> 1;
        if (a.lin[mid].cum_weight <= (uint64_t)b) li = mid; else hi = mid - 1;
    }
    const LinDesc& L = a.lin[li];
    const long wg = (long)b - (long)L.cum_weight;          // split-major: a split's groups are neighbours
    const int row_blocks = rows_row_blocks(L, a.row_tiles);
    const long rb = wg % row_blocks;
    const int split = (int)(wg / row_blocks);
    float* partial = a.partial + L.step_weight;
    switch (L.variant) {
    case V_W3: run_rows<V_W3, WAVES, TILES, MT>(L, a.M, rb, split, partial, red); break;
    case V_W4: run_rows<V_W4, WAVES, TILES, MT>(L, a.M, rb, split, partial, red); break;
    case V_W8: run_rows<V_W8, WAVES, TILES, MT>(L, a.M, rb, split, partial, red); break;
    case V_I8: run_rows<V_I8, WAVES, TILES, MT>(L, a.M, rb, split, partial, red); break;
    default:   run_rows<V_F16, WAVES, TILES, MT>(L, a.M, rb, split, partial, red); break;
    }
}

// Second kernel of a K-split linear of a small launch: adds the splits in order, then bias, activation,
// residual and the one rounding; four consecutive rows of one token per thread.
__global__ __launch_bounds__(256) void decode_rows_reduce_kernel(const DecodeArgs a, int li)
{
    const LinDesc& L = a.lin[li];
    const float* __restrict__ partial = a.partial + L.step_weight;
    const size_t quads = (size_t)a.M * L.N / 4, plane = (size_t)(a.M <= 16 ? 16 : 32) * L.N;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < quads; q += (size_t)gridDim.x * 256) {
        const size_t e = 4 * q;
        const int n = (int)(e % L.N);
        f4 sum = *reinterpret_cast<const f4*>(partial + e);
        for (int sp = 1; sp < L.aux; ++sp) sum += *reinterpret_cast<const f4*>(partial + sp * plane + e);
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

}  // namespace

}  // namespace lpq

// Scratch of the entry point that allocates nothing (lpq_stage_linears_noalloc): what the library otherwise keeps in
// its growing workspace -- the fp32 partial tiles of the launches and the prepared activations of a decode launch.
// 128 MiB per device, held until the process ends.  A decode launch of up to 32 token rows takes 32 MiB of partial
// tiles (2 slots x 256 workgroups x 32 rows x 512 columns x 4 bytes), group sums (48 linears of K = 57344: 2.7 MiB)
// and, at up to 16 rows, 2 bytes per token row and column of scaled activations for 3-bit linears read in place (ten
// BLOOM-176B-shaped layers at 16 rows: 31 MiB); passes of 64 rows take 64 MiB of partial tiles.  Nothing in it has to
// start at zero:
// whatever is read was written earlier in the same call.
constexpr size_t LPQ_SCRATCH_BYTES = (size_t)128 << 20;
static __device__ __align__(256) unsigned char scratch[LPQ_SCRATCH_BYTES];

namespace lpq {

// In host code `scratch` is only a handle for the symbol; its address on the current device comes from the runtime,
// once per device (each device has its own copy of the array).
hipError_t static_scratch(void** ptr, size_t* bytes)
{
    static std::mutex mu;
    static void* addr[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    *bytes = LPQ_SCRATCH_BYTES;
    return hipSuccess;
}

template <int TOK, int WAVES, int CAP>
static hipError_t launch_tok(const DecodeArgs& a, hipStream_t s)
{
    // the slab may exceed the 64 KB that needs no opt-in: raise the kernel's limit once per device
    static std::once_flag flags[64];
    static hipError_t results[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::call_once(flags[dev], [&] {
        results[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<TOK, WAVES, CAP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(DecodeSmem<TOK, WAVES, CAP>));
    });
    if (results[dev] != hipSuccess) return results[dev];
    decode_kernel<TOK, WAVES, CAP><<<(unsigned)a.n_blocks, 64 * WAVES, sizeof(DecodeSmem<TOK, WAVES, CAP>), s>>>(a);
    return hipGetLastError();
}

template <int WAVES>
static hipError_t launch_waves(const DecodeArgs& a, hipStream_t s)
{
    const int rows = a.M - a.m0;
    if (rows > 32) return launch_tok<64, WAVES, 8>(a, s);
    if (rows > 16) return launch_tok<32, WAVES, 8>(a, s);
    // Up to 16 token rows the LDS holds two buffers of 16 steps.  The longer chunk halves the workgroup barriers (2-3 %
    // on a 3-bit stage of K = 14336 and 57344), but a linear's K then has to be whole or half chunks: any other
    // remainder runs in the conditional form of the main loop, which costs more than the barriers saved.
    bool whole = true;
    for (int li = 0; li < a.n_lin; ++li) whole = whole && a.lin[li].kt % 8 == 0;
    return whole ? launch_tok<16, WAVES, 16>(a, s) : launch_tok<16, WAVES, 8>(a, s);
}

hipError_t launch_decode_rows(const DecodeArgs& a, hipStream_t s)
{
    const unsigned grid = (unsigned)a.n_blocks;
#define LPQ_ROWS_CASE(T)                                                                      \
    case T:                                                                                   \
        if (a.M > 16)          decode_rows_kernel<4, T, 2><<<grid, 256, 0, s>>>(a);           \
        else if (a.waves == 8) decode_rows_kernel<8, T, 1><<<grid, 512, 0, s>>>(a);           \
        else                   decode_rows_kernel<4, T, 1><<<grid, 256, 0, s>>>(a);           \
        break;
    if (a.M > 32) return hipErrorInvalidValue;
    switch (a.row_tiles) {
        LPQ_ROWS_CASE(2) LPQ_ROWS_CASE(3) LPQ_ROWS_CASE(4) LPQ_ROWS_CASE(5)
    default: return hipErrorInvalidValue;
    }
#undef LPQ_ROWS_CASE
    hipError_t e = hipGetLastError();
    for (int li = 0; li < a.n_lin && e == hipSuccess; ++li) {
        if (a.lin[li].aux <= 1) continue;
        const size_t quads = (size_t)a.M * a.lin[li].N / 4;
        decode_rows_reduce_kernel<<<(unsigned)std::min<size_t>((quads + 255) / 256, 4096), 256, 0, s>>>(a, li);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_decode(const DecodeArgs& a, hipStream_t s)
{
    if (a.waves != 8) return hipErrorInvalidValue;
    const int rows = a.M - a.m0;
    if (rows <= 32) {       // the kernels for up to 32 token rows take the zero term from the activations' group sums
        bool any = false;
        for (int li = 0; li < a.n_lin; ++li) any = any || a.lin[li].variant != V_F16;
        if (any) {
            if (!a.prep) return hipErrorInvalidValue;
            bool inplace = false;
            for (int li = 0; li < a.n_lin; ++li) inplace = inplace || a.lin[li].variant == V_W3_INPLACE;
            const dim3 grid((unsigned)a.n_lin, (unsigned)rows);
            if (inplace) decode_prepare_kernel<true><<<grid, GS_THREADS, 0, s>>>(a, const_cast<uint16_t*>(a.prep));
            else         decode_prepare_kernel<false><<<grid, GS_THREADS, 0, s>>>(a, const_cast<uint16_t*>(a.prep));
            const hipError_t e0 = hipGetLastError();
            if (e0 != hipSuccess) return e0;
        }
    }
    hipError_t e = launch_waves<8>(a, s);
    if (e != hipSuccess) return e;
    if (a.n_blocks > 1) {
        const int m_cnt = std::min(64, a.M - a.m0);
        const dim3 grid((unsigned)(a.n_blocks - 1), (unsigned)((m_cnt * a.waves * 16 + 1023) / 1024));     // passes of 1024 groups of 4 rows
        decode_fixup_kernel<<<grid, 256, 0, s>>>(a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace lpq
