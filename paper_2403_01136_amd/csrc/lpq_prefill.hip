// Prefill-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for M = eta * s prompt tokens (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the prefill phase is bound by FLOPs;
// Sec. 4.3: prefill micro-batch eta, prompt length s).
//
// A workgroup of four wavefronts computes a BM x 256 block of y.  Each wave owns one 64-row
// block of W (four 16-row tiles) for all BM tokens, so packed weight tiles go straight from
// global memory into that wave's registers in MFMA operand order, are dequantised there once per
// 128-column step (scale * code + zero, one fp16 rounding) and never touch LDS.  The activations
// of the block are shared by the four waves through a double-buffered, padded LDS slab.
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

template <int BM> struct PrefillSmem {
    enum { ROW_HALVES = 128 + 8 };                 // +16 bytes per row: conflict-free 16-byte operand reads
    uint16_t x[2][BM][ROW_HALVES];
};

template <int V, int BM>
__global__ __launch_bounds__(256) void prefill_kernel(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                      const uint16_t* __restrict__ zeros, const uint16_t* __restrict__ x,
                                                      uint16_t* __restrict__ y, const uint16_t* __restrict__ bias,
                                                      int M, int K, int N)
{
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr int NW = 4;                           // 16-row tiles per wave = one 64-row block
    constexpr int MTB = BM / 16;                    // token tiles per block
    constexpr int XV = BM * 128 / 8 / 256;          // 16-byte pieces of the x slab per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    PrefillSmem<BM>& sm = *reinterpret_cast<PrefillSmem<BM>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int KT = K / 128;
    const long RB = N / 64;                          // 64-row blocks of W
    const int m0 = blockIdx.y * BM;
    const long rb = (long)blockIdx.x * 4 + wave;     // this wave's row block
    const bool active = rb < RB;                     // idle waves still stage activations
    const long rbc = active ? rb : RB - 1;

    f4 acc[NW][MTB];
#pragma unroll
    for (int t = 0; t < NW; ++t)
#pragma unroll
        for (int mt = 0; mt < MTB; ++mt) acc[t][mt] = f4{0, 0, 0, 0};

    // x slab: piece p = tid + 256*i covers token row p/16, 8 halves at column 8*(p%16)
    u32x4 xr[XV];
    auto load_x_slab = [&](int kt) {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = tid + 256 * i, row = p >> 4, col = (p & 15) * 8;
            const int tok = m0 + row;
            u32x4 v = {0, 0, 0, 0};
            if (tok < M) v = *reinterpret_cast<const u32x4*>(x + (long)tok * K + (long)kt * 128 + col);
            xr[i] = v;
        }
    };
    auto store_x_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = tid + 256 * i, row = p >> 4, col = (p & 15) * 8;
            *reinterpret_cast<u32x4*>(&sm.x[buf][row][col]) = xr[i];
        }
    };
    WRaw<V> wraw[NW];
    u32x2 ws, wz;                                    // fp16 scale / zero of the lane's four rows 4r..4r+3
    auto load_w = [&](int kt) {
#pragma unroll
        for (int t = 0; t < NW; ++t) wraw[t] = load_tile<V>(codes, rbc, KT, kt, t, lane);
        if constexpr (SCHEME == SCH_ASYM) {
            const size_t idx = (size_t)kt * N + rbc * 64 + 4 * r;
            ws = *reinterpret_cast<const u32x2*>(scales + idx);
            wz = *reinterpret_cast<const u32x2*>(zeros + idx);
        }
    };

    load_x_slab(0);
    load_w(0);
    store_x_slab(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        // dequantise this step's weight tiles, then start the next step's loads
        h8 wb[NW][4];
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            unpack_codes<V>(wraw[t], wb[t]);
            if constexpr (SCHEME == SCH_ASYM) {
                const uint32_t sp = ws[t >> 1], zp = wz[t >> 1];
                const uint16_t sh = (uint16_t)((t & 1) ? (sp >> 16) : (sp & 0xffffu));
                const uint16_t zh = (uint16_t)((t & 1) ? (zp >> 16) : (zp & 0xffffu));
                apply_scale_zero(wb[t], __builtin_bit_cast(_Float16, sh), __builtin_bit_cast(_Float16, zh));
            }
        }
        if (kt + 1 < KT) { load_x_slab(kt + 1); load_w(kt + 1); }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MTB; ++mt) {
                const h8 a = *reinterpret_cast<const h8*>(&sm.x[buf][16 * mt + r][32 * j + 8 * kq]);
#pragma unroll
                for (int t = 0; t < NW; ++t) acc[t][mt] = mfma16(a, wb[t][j], acc[t][mt]);
            }
        if (kt + 1 < KT) store_x_slab(buf ^ 1);
        __syncthreads();
    }

    if (!active) return;
    // epilogue: lane holds tokens 4*kq + v of the four consecutive rows 64*rb + 4*r + t
    const long nbase = rb * 64 + 4 * r;
    float post[NW], bs[NW];
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        post[t] = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post[t] = (float)__builtin_bit_cast(_Float16, scales[nbase + t]);
        bs[t] = bias ? (float)__builtin_bit_cast(_Float16, bias[nbase + t]) : 0.0f;
    }
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tok = m0 + 16 * mt + 4 * kq + v;
            if (tok >= M) continue;
            h4 o;
#pragma unroll
            for (int t = 0; t < NW; ++t) o[t] = (_Float16)(acc[t][mt][v] * post[t] + bs[t]);
            *reinterpret_cast<h4*>(y + (size_t)tok * N + nbase) = o;
        }
}

template <int V>
hipError_t launch_variant(const lpq_qweight& w, const void* x, int M, void* y, hipStream_t s)
{
    constexpr int BM = 128, BN = 256;
    const dim3 grid((unsigned)((w.d.N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    const size_t smem = sizeof(PrefillSmem<BM>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<V, BM>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    prefill_kernel<V, BM><<<grid, 256, smem, s>>>(
        static_cast<const uint8_t*>(w.codes), static_cast<const uint16_t*>(w.scales), static_cast<const uint16_t*>(w.zeros),
        static_cast<const uint16_t*>(x), static_cast<uint16_t*>(y), static_cast<const uint16_t*>(w.bias), M, w.d.K, w.d.N);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill(const lpq_qweight& w, const void* x, int M, void* y, hipStream_t s)
{
    switch (variant_of(w.d)) {
    case V_W3: return launch_variant<V_W3>(w, x, M, y, s);
    case V_W4: return launch_variant<V_W4>(w, x, M, y, s);
    case V_W8: return launch_variant<V_W8>(w, x, M, y, s);
    case V_I8: return launch_variant<V_I8>(w, x, M, y, s);
    case V_F16: return launch_variant<V_F16>(w, x, M, y, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lpq
