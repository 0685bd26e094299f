// Prefill-phase linears: y[M][N] = x[M][K] . w~[N][K]^T for M = eta * s prompt tokens (LLM-PQ,
// arXiv 2403.01136, Sec. 4.1 "Latency Cost Model": the prefill phase is bound by FLOPs;
// Sec. 4.3: prefill micro-batch eta, prompt length s).
//
// A workgroup of four wavefronts computes a BM x BN block of y.  Each wave owns NW 16-row
// weight tiles (its own slice of BN) for all BM tokens, so packed weight tiles go straight from
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

template <int V, int BM, int NW>
__global__ __launch_bounds__(256) void prefill_kernel(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                      const uint16_t* __restrict__ zeros, const uint16_t* __restrict__ x,
                                                      uint16_t* __restrict__ y, const uint16_t* __restrict__ bias,
                                                      int M, int K, int N)
{
    constexpr int SCHEME = VInfo<V>::SCHEME;
    constexpr int MTB = BM / 16;                    // token tiles per block
    constexpr int XV = BM * 128 / 8 / 256;          // 16-byte pieces of the x slab per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    PrefillSmem<BM>& sm = *reinterpret_cast<PrefillSmem<BM>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int KT = K / 128;
    const long NT = N / 16;
    const int m0 = blockIdx.y * BM;
    const long nt0 = ((long)blockIdx.x * 4 + wave) * NW;

    long ntc[NW];
#pragma unroll
    for (int rt = 0; rt < NW; ++rt) ntc[rt] = min(nt0 + rt, NT - 1);

    f4 acc[NW][MTB];
#pragma unroll
    for (int rt = 0; rt < NW; ++rt)
#pragma unroll
        for (int mt = 0; mt < MTB; ++mt) acc[rt][mt] = f4{0, 0, 0, 0};

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
    uint16_t ws[NW], wz[NW];
    auto load_w = [&](int kt) {
#pragma unroll
        for (int rt = 0; rt < NW; ++rt) {
            wraw[rt] = load_tile<V>(codes, ntc[rt], KT, kt, lane);
            if constexpr (SCHEME == SCH_ASYM) {
                const long idx = (ntc[rt] * 16 + r) * KT + kt;
                ws[rt] = scales[idx];
                wz[rt] = zeros[idx];
            }
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
        for (int rt = 0; rt < NW; ++rt) {
            unpack_codes<V>(wraw[rt], wb[rt]);
            if constexpr (SCHEME == SCH_ASYM)
                apply_scale_zero(wb[rt], __builtin_bit_cast(_Float16, ws[rt]), __builtin_bit_cast(_Float16, wz[rt]));
        }
        if (kt + 1 < KT) { load_x_slab(kt + 1); load_w(kt + 1); }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MTB; ++mt) {
                const h8 a = *reinterpret_cast<const h8*>(&sm.x[buf][16 * mt + r][32 * j + 8 * kq]);
#pragma unroll
                for (int rt = 0; rt < NW; ++rt) acc[rt][mt] = mfma16(a, wb[rt][j], acc[rt][mt]);
            }
        if (kt + 1 < KT) store_x_slab(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int rt = 0; rt < NW; ++rt) {
        if (nt0 + rt >= NT) continue;
        const long n = (nt0 + rt) * 16 + r;
        float post = 1.0f;
        if constexpr (SCHEME == SCH_SYM) post = (float)__builtin_bit_cast(_Float16, scales[n]);
        const float b = bias ? (float)__builtin_bit_cast(_Float16, bias[n]) : 0.0f;
#pragma unroll
        for (int mt = 0; mt < MTB; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = m0 + 16 * mt + 4 * kq + v;
                if (tok < M) y[(long)tok * N + n] = __builtin_bit_cast(uint16_t, (_Float16)(acc[rt][mt][v] * post + b));
            }
    }
}

template <int V>
hipError_t launch_variant(const lpq_qweight& w, const void* x, int M, void* y, hipStream_t s)
{
    constexpr int BM = 128, NW = 4, BN = 4 * NW * 16;
    const dim3 grid((unsigned)((w.d.N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    const size_t smem = sizeof(PrefillSmem<BM>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<V, BM, NW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    prefill_kernel<V, BM, NW><<<grid, 256, smem, s>>>(
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
