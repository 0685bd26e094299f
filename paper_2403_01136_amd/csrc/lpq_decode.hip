// Decode-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for a small micro-batch M (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the decode phase is bound by the bytes it
// streams; Sec. 4.3: M = xi, one token per sequence).
//
// One grouped launch covers every linear of a stage.  A work unit is (linear, block of W rows,
// K range); one wavefront owns one unit, streams its packed tiles from HBM with 16-byte (12-byte
// for 3-bit) per-lane loads that are contiguous across the wave, unpacks them in registers into
// MFMA B operands and multiplies them with the activations held as A operands.  Units whose K
// range is the whole of K write fp16 outputs directly; otherwise they write fp32 partial sums and
// a second small kernel adds them in a fixed order (deterministic results).
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

template <int V> struct DecodeCfg { enum { RT = (V == V_F16) ? 2 : 4 }; };   // 16-row tiles per unit

// activations of one 128-column tile as MFMA A operands: xa[mt][j]
template <int MT>
__device__ __forceinline__ void load_x(const uint16_t* __restrict__ x, int K, int M, int m0, int kt, int lane, h8 xa[MT][4])
{
    const int i = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int tok = m0 + 16 * mt + i;
        const uint16_t* p = x + (long)tok * K + (long)kt * 128 + 8 * kq;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            h8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (tok < M) v = *reinterpret_cast<const h8*>(p + 32 * j);
            xa[mt][j] = v;
        }
    }
}

template <int V, int MT>
__device__ __forceinline__ void run_unit(const LinDesc& L, int M, int m0, int unit, int lane)
{
    constexpr int RT = DecodeCfg<V>::RT;
    constexpr int SCHEME = VInfo<V>::SCHEME;
    const int KT = L.K / 128;
    const int rg = unit % L.row_groups, split = unit / L.row_groups;
    const long nt0 = (long)rg * RT;
    const long NT = L.N / 16;
    const int kt_begin = split * L.kt_per_split;
    const int kt_end = min(KT, kt_begin + L.kt_per_split);
    const int r = lane & 15;

    f4 acc[RT][MT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = f4{0, 0, 0, 0};

    // row tiles past the end of W are clamped to the last tile for loads and dropped at the store
    long ntc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) ntc[rt] = min(nt0 + rt, NT - 1);

    WRaw<V> cur[RT], nxt[RT];
    uint16_t cs[RT], cz[RT], ns[RT], nz[RT];
    auto fetch = [&](int kt, WRaw<V> w[RT], uint16_t s[RT], uint16_t z[RT]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            w[rt] = load_tile<V>(L.codes, ntc[rt], KT, kt, lane);
            if constexpr (SCHEME == SCH_ASYM) {
                const long idx = (ntc[rt] * 16 + r) * KT + kt;
                s[rt] = L.scales[idx];
                z[rt] = L.zeros[idx];
            }
        }
    };
    fetch(kt_begin, cur, cs, cz);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const int ktn = min(kt + 1, kt_end - 1);
        fetch(ktn, nxt, ns, nz);
        h8 xa[MT][4];
        load_x<MT>(L.x, L.K, M, m0, kt, lane, xa);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            h8 wb[4];
            unpack_codes<V>(cur[rt], wb);
            if constexpr (SCHEME == SCH_ASYM)
                apply_scale_zero(wb, __builtin_bit_cast(_Float16, cs[rt]), __builtin_bit_cast(_Float16, cz[rt]));
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = mfma16(xa[mt][j], wb[j], acc[rt][mt]);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) { cur[rt] = nxt[rt]; cs[rt] = ns[rt]; cz[rt] = nz[rt]; }
    }

    // epilogue: lane holds tokens 4*(lane/16)+v of output row n = 16*nt + lane%16
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        if (nt0 + rt >= NT) continue;
        const long n = (nt0 + rt) * 16 + r;
        float post = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post = (float)__builtin_bit_cast(_Float16, L.scales[n]);
        const float b = (L.bias && L.ksplit == 1) ? (float)__builtin_bit_cast(_Float16, L.bias[n]) : 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = m0 + 16 * mt + 4 * (lane >> 4) + v;
                if (tok >= M) continue;
                const float val = acc[rt][mt][v] * post;
                if (L.ksplit == 1) L.y[(long)tok * L.N + n] = __builtin_bit_cast(uint16_t, (_Float16)(val + b));
                else L.partial[((long)split * M + tok) * L.N + n] = val;
            }
    }
}

template <int MT>
__global__ __launch_bounds__(256) void decode_kernel(const DecodeArgs a)
{
    const int unit_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit_global >= a.total_units) return;
    const int lane = threadIdx.x & 63;
    int li = 0;
    while (li + 1 < a.n_lin && a.lin[li + 1].unit_begin <= unit_global) ++li;
    const LinDesc& L = a.lin[li];
    const int unit = unit_global - L.unit_begin;
    switch (L.variant) {
    case V_W3: run_unit<V_W3, MT>(L, a.M, a.m0, unit, lane); break;
    case V_W4: run_unit<V_W4, MT>(L, a.M, a.m0, unit, lane); break;
    case V_W8: run_unit<V_W8, MT>(L, a.M, a.m0, unit, lane); break;
    case V_I8: run_unit<V_I8, MT>(L, a.M, a.m0, unit, lane); break;
    default:   run_unit<V_F16, MT>(L, a.M, a.m0, unit, lane); break;
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
    for (int k = 0; k < L.ksplit; ++k) s += *reinterpret_cast<const f4*>(L.partial + ((long)k * a.M + tok) * L.N + n);
    if (L.bias)
#pragma unroll
        for (int v = 0; v < 4; ++v) s[v] += (float)__builtin_bit_cast(_Float16, L.bias[n + v]);
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    h4 o = {(_Float16)s[0], (_Float16)s[1], (_Float16)s[2], (_Float16)s[3]};
    *reinterpret_cast<h4*>(L.y + (long)tok * L.N + n) = o;
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, int n_red_blocks, hipStream_t s)
{
    const int rows = a.M - a.m0;
    const unsigned blocks = (unsigned)((a.total_units + 3) / 4);
    if (rows <= 16)      decode_kernel<1><<<blocks, 256, 0, s>>>(a);
    else if (rows <= 32) decode_kernel<2><<<blocks, 256, 0, s>>>(a);
    else if (rows <= 48) decode_kernel<3><<<blocks, 256, 0, s>>>(a);
    else                 decode_kernel<4><<<blocks, 256, 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (n_red_blocks > 0) {
        splitk_reduce_kernel<<<(unsigned)n_red_blocks, 256, 0, s>>>(a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace lpq
