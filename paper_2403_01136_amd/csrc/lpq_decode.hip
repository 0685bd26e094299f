// Decode-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for a small micro-batch M (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the decode phase is bound by the bytes it
// streams; Sec. 4.3: M = xi, one token per sequence).
//
// One grouped launch covers every linear of a stage.  A work unit is (linear, K range, 4
// consecutive row blocks); one workgroup of four wavefronts owns a unit and each wave owns one
// row block (64 rows of W; 32 for fp16 weights).  A wave streams its block's packed tiles from
// HBM as one sequential stream of 16-byte (12-byte for 3-bit) per-lane loads that are contiguous
// across the wave, keeps several 128-column steps in flight in registers, unpacks them there into
// MFMA B operands and multiplies them with the activations (MFMA A operands).  The activations of
// the unit's K range are staged once per workgroup through a double-buffered LDS slab, so they
// cost a quarter of the global loads they would cost per wave.  Units whose K range is the whole
// of K write fp16 outputs directly; otherwise they write fp32 partial sums and a second small
// kernel adds them in a fixed order (deterministic results).
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

// RT: 16-row tiles per wave.  DEPTH: 128-column steps of weights a wave keeps in flight (a step is
// 3-4 KB per wave for 3/4-bit codes and 8 KB for 8-bit codes and fp16 rows, so 12-16 KB either way).
template <int V> struct DecodeCfg { enum { RT = (V == V_F16) ? 2 : 4, DEPTH = (V == V_W3 || V == V_W4) ? 4 : 2 }; };

// activation staging: CHUNK 128-column steps per LDS buffer
template <int MT> struct PipeCfg {
    enum { CHUNK = (MT == 1) ? 8 : (MT == 2) ? 4 : 2 };
    enum { ROW_HALVES = CHUNK * 128 + 8 };          // +16 bytes: conflict-free 16-byte operand reads
    enum { PIECES = MT * CHUNK };                   // 16-byte pieces of a chunk per thread (256 threads)
};

template <int MT> struct DecodeSmem { uint16_t x[2][16 * MT][PipeCfg<MT>::ROW_HALVES]; };

template <int V, int MT>
__device__ __forceinline__ void run_unit(const LinDesc& L, int M, int m0, int unit, DecodeSmem<MT>& sm)
{
    constexpr int RT = DecodeCfg<V>::RT;
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr int CHUNK = PipeCfg<MT>::CHUNK, PIECES = PipeCfg<MT>::PIECES;
    constexpr int STAGES = DecodeCfg<V>::DEPTH < CHUNK ? DecodeCfg<V>::DEPTH : CHUNK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int KT = L.K / 128;
    const int sb = unit % L.row_superblocks, split = unit / L.row_superblocks;
    const long rb = (long)sb * 4 + wave;                  // this wave's row block
    const bool active = rb < L.row_blocks;                // idle waves still stage activations
    const long rbc = active ? rb : L.row_blocks - 1;
    const int kt_begin = split * L.kt_per_split;
    const int kt_end = min(KT, kt_begin + L.kt_per_split);

    f4 acc[RT][MT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = f4{0, 0, 0, 0};

    // ---- weight pipeline: one Stage = everything one 128-column step needs from global memory
    struct Stage {
        WRaw<V> w[RT];
        u32x2 s, z;          // fp16 scale / zero of the lane's four rows (tiles 0..3), grouped scheme only
    };
    Stage st[STAGES];
    auto issue = [&](Stage& b, int kt) {
        kt = min(kt, kt_end - 1);
        if constexpr (RT == 4) {
#pragma unroll
            for (int t = 0; t < RT; ++t) b.w[t] = load_tile<V>(L.codes, rbc, KT, kt, t, lane);
        } else {   // half a 64-row block per wave: tiles 2*(rbc%2) + t
#pragma unroll
            for (int t = 0; t < RT; ++t) b.w[t] = load_tile<V>(L.codes, rbc >> 1, KT, kt, 2 * (int)(rbc & 1) + t, lane);
        }
        if constexpr (SCHEME == SCH_ASYM) {
            const size_t idx = (size_t)kt * L.N + rbc * 64 + 4 * r;
            b.s = *reinterpret_cast<const u32x2*>(L.scales + idx);
            b.z = *reinterpret_cast<const u32x2*>(L.zeros + idx);
        }
    };
    // Two ways to fold scale and zero in.  POST (few tokens): multiply raw codes on the matrix
    // cores per 128-column group, then acc += scale * (codes . x) + zero * sum(x) in fp32, with
    // sum(x) from one extra MFMA against a block of ones -- the scale costs 8 fp32 FMAs per tile
    // instead of 16 packed FMAs plus the int -> fp16 conversions.  Otherwise (many tokens, where the
    // fp32 work would grow with M): dequantise each weight to fp16 once, w~ = scale * code + zero.
    constexpr bool POST = (MT <= 2) && V != V_F16;
    f4 xsum[MT];                      // per-row scheme only: sum of x over the whole K range
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xsum[mt] = f4{0, 0, 0, 0};
    auto compute = [&](Stage& b, int buf, int step) {
        h8 wb[RT][4];
        if constexpr (POST) {
#pragma unroll
            for (int t = 0; t < RT; ++t) unpack_subnormal<V>(b.w[t], wb[t]);
            const _Float16 one = (_Float16)1.0f;
            const h8 ones = {one, one, one, one, one, one, one, one};
            if constexpr (SCHEME == SCH_ASYM) {
                f4 d[RT][MT], xs[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    xs[mt] = f4{0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < RT; ++t) d[t][mt] = f4{0, 0, 0, 0};
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const h8 a = *reinterpret_cast<const h8*>(&sm.x[buf][16 * mt + r][step * 128 + 32 * j + 8 * kq]);
                        xs[mt] = mfma16(a, ones, xs[mt]);
#pragma unroll
                        for (int t = 0; t < RT; ++t) d[t][mt] = mfma16(a, wb[t][j], d[t][mt]);
                    }
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    const uint32_t sp = b.s[t >> 1], zp = b.z[t >> 1];
                    const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                    const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                    const float sf = (float)__builtin_bit_cast(_Float16, sh) * 16777216.0f;     // scale * 2^24
                    const float zf = (float)__builtin_bit_cast(_Float16, zh);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            acc[t][mt][v] = __builtin_fmaf(sf, d[t][mt][v], __builtin_fmaf(zf, xs[mt][v], acc[t][mt][v]));
                }
            } else {   // per-row scheme: one scale per row, applied in the epilogue
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const h8 a = *reinterpret_cast<const h8*>(&sm.x[buf][16 * mt + r][step * 128 + 32 * j + 8 * kq]);
                        xsum[mt] = mfma16(a, ones, xsum[mt]);
#pragma unroll
                        for (int t = 0; t < RT; ++t) acc[t][mt] = mfma16(a, wb[t][j], acc[t][mt]);
                    }
            }
        } else {
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
                    const h8 a = *reinterpret_cast<const h8*>(&sm.x[buf][16 * mt + r][step * 128 + 32 * j + 8 * kq]);
#pragma unroll
                    for (int t = 0; t < RT; ++t) acc[t][mt] = mfma16(a, wb[t][j], acc[t][mt]);
                }
        }
    };

    // ---- activation staging: chunk c covers steps [kt_begin + c*CHUNK, +CHUNK)
    u32x4 xr[PIECES];
    auto load_x_chunk = [&](int kt0) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int p = tid + 256 * i, row = p / (CHUNK * 16), c16 = p % (CHUNK * 16);
            const int tok = m0 + row, col = kt0 * 128 + c16 * 8;
            u32x4 v = {0, 0, 0, 0};
            if (tok < M && col < kt_end * 128) v = *reinterpret_cast<const u32x4*>(L.x + (size_t)tok * L.K + col);
            xr[i] = v;
        }
    };
    auto store_x_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int p = tid + 256 * i, row = p / (CHUNK * 16), c16 = p % (CHUNK * 16);
            *reinterpret_cast<u32x4*>(&sm.x[buf][row][c16 * 8]) = xr[i];
        }
    };

    load_x_chunk(kt_begin);
    if (active) {
#pragma unroll
        for (int s = 0; s < STAGES; ++s) issue(st[s], kt_begin + s);
    }
    store_x_chunk(0);
    __syncthreads();
    int buf = 0;
    for (int kt = kt_begin; kt < kt_end; kt += CHUNK) {
        const bool more = kt + CHUNK < kt_end;
        if (more) load_x_chunk(kt + CHUNK);
        if (active) {
#pragma unroll
            for (int s = 0; s < CHUNK; ++s) {
                if (kt + s < kt_end) {
                    compute(st[s % STAGES], buf, s);
                    issue(st[s % STAGES], kt + s + STAGES);
                }
            }
        }
        if (more) store_x_chunk(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    if (!active) return;

    // ---- epilogue: lane holds tokens 4*kq + v of RT consecutive rows starting at nbase
    const long nbase = (RT == 4) ? rb * 64 + 4 * r : (rb >> 1) * 64 + 4 * r + 2 * (rb & 1);
    float post[RT], bias[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        post[t] = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post[t] = (float)__builtin_bit_cast(_Float16, L.scales[nbase + t]);
        bias[t] = (L.bias && L.ksplit == 1) ? (float)__builtin_bit_cast(_Float16, L.bias[nbase + t]) : 0.0f;
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
                float a = acc[t][mt][v];
                if constexpr (POST && SCHEME == SCH_SYM) a = a * 16777216.0f - 128.0f * xsum[mt][v];   // undo 2^-24 and the +128 offset
                val[t] = a * post[t];
            }
            if (L.ksplit == 1) {
                typedef _Float16 hv __attribute__((ext_vector_type(RT)));
                hv o;
#pragma unroll
                for (int t = 0; t < RT; ++t) o[t] = (_Float16)(val[t] + bias[t]);
                *reinterpret_cast<hv*>(L.y + (size_t)tok * L.N + nbase) = o;
            } else {
                typedef float fv __attribute__((ext_vector_type(RT)));
                fv o;
#pragma unroll
                for (int t = 0; t < RT; ++t) o[t] = val[t];
                *reinterpret_cast<fv*>(L.partial + ((size_t)split * M + tok) * L.N + nbase) = o;
            }
        }
}

template <int MT>
__global__ __launch_bounds__(256, 2) void decode_kernel(const DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    DecodeSmem<MT>& sm = *reinterpret_cast<DecodeSmem<MT>*>(smem_raw);
    const int unit_global = blockIdx.x;
    int li = 0;
    while (li + 1 < a.n_lin && a.lin[li + 1].unit_begin <= unit_global) ++li;
    const LinDesc& L = a.lin[li];
    const int unit = unit_global - L.unit_begin;
    switch (L.variant) {
    case V_W3: run_unit<V_W3, MT>(L, a.M, a.m0, unit, sm); break;
    case V_W4: run_unit<V_W4, MT>(L, a.M, a.m0, unit, sm); break;
    case V_W8: run_unit<V_W8, MT>(L, a.M, a.m0, unit, sm); break;
    case V_I8: run_unit<V_I8, MT>(L, a.M, a.m0, unit, sm); break;
    default:   run_unit<V_F16, MT>(L, a.M, a.m0, unit, sm); break;
    }
}

// y[m][n] = fp16(sum_s partial[s][m][n] + bias[n]), s ascending; 256 threads x 4 columns per block
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const DecodeArgs a)
{
    int li = -1;
    for (int i = 0; i < a.n_lin; ++i)
        if (a.lin[i].ksplit > 1 && a.lin[i].red_begin <= (int)blockIdx.x) li = i;
    if (li < 0) return;
    const LinDesc& L = a.lin[li];
    const int m_lo = a.m0, m_cnt = min(64, a.M - a.m0);
    const long per_row = L.N / 4;
    const long idx = ((long)blockIdx.x - L.red_begin) * 256 + threadIdx.x;
    if (idx >= per_row * m_cnt) return;
    const int tok = m_lo + (int)(idx / per_row);
    const long n = (idx % per_row) * 4;
    f4 s = {0, 0, 0, 0};
    for (int k = 0; k < L.ksplit; ++k) s += *reinterpret_cast<const f4*>(L.partial + ((size_t)k * a.M + tok) * L.N + n);
    if (L.bias)
#pragma unroll
        for (int v = 0; v < 4; ++v) s[v] += (float)__builtin_bit_cast(_Float16, L.bias[n + v]);
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    h4 o = {(_Float16)s[0], (_Float16)s[1], (_Float16)s[2], (_Float16)s[3]};
    *reinterpret_cast<h4*>(L.y + (size_t)tok * L.N + n) = o;
}

}  // namespace

template <int MT>
static hipError_t launch_mt(const DecodeArgs& a, hipStream_t s)
{
    static bool attr_set = false;      // the slab is just over the 64 KB that needs no opt-in
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<MT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(DecodeSmem<MT>));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    decode_kernel<MT><<<(unsigned)a.total_units, 256, sizeof(DecodeSmem<MT>), s>>>(a);
    return hipGetLastError();
}

hipError_t launch_decode(const DecodeArgs& a, int n_red_blocks, hipStream_t s)
{
    const int rows = a.M - a.m0;
    hipError_t e = rows <= 16 ? launch_mt<1>(a, s) : rows <= 32 ? launch_mt<2>(a, s) : rows <= 48 ? launch_mt<3>(a, s) : launch_mt<4>(a, s);
    if (e != hipSuccess) return e;
    if (n_red_blocks > 0) {
        splitk_reduce_kernel<<<(unsigned)n_red_blocks, 256, 0, s>>>(a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace lpq
