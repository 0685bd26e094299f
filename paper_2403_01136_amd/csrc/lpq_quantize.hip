// Round-to-nearest quantiser + bit-packer, and the unpack/dequantise test helper.
//
// LLM-PQ (arXiv 2403.01136) Sec. 2.4: s = (max - min) / (2^b - 1), code = round((w - q) / s)
// with q = min; Sec. 4.2: symmetric scaling factor max|w| / (2^(b-1) - 1) for the per-row
// scheme; Sec. 4.1: dense packing, bit/8 bytes per weight.
//
// One wavefront quantises one 16x128 tile (tile t of a 64-row block holds rows 4*r + t).  Lane
// (r = lane%16, kq = lane/16) reads exactly the 32 weights it owns in the packed format (four
// 16-byte pieces of its row), so min/max need one exchange across the four kq lanes of a row and
// the packing itself is lane-local.  The four waves of a workgroup take the four tiles of a block.
// All fp32 steps use the round-to-nearest intrinsics so the compiler can neither fuse nor
// reassociate them: the results are bit-exact functions of the input.
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

// The 64-row blocks [rb0, rb0 + n_rb) of W that a launch quantises; the source pointer starts at row 64 * rb0.
struct RowWindow { long rb0, n_rb; };

__device__ __forceinline__ uint16_t f2h_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
__device__ __forceinline__ float h2f_bits(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// the lane's 32 weights of its row n in 128-column step kt: v[8*j + e] = W[n][128*kt + 32*j + 8*kq + e]
__device__ __forceinline__ void load_owned(const uint16_t* __restrict__ w, long K, long n, int kt, int lane, float v[32])
{
    const int kq = lane >> 4;
    const uint16_t* p = w + n * K + (long)kt * 128 + 8 * kq;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const h8 t = *reinterpret_cast<const h8*>(p + 32 * j);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[8 * j + e] = (float)t[e];
    }
}

template <int BITS, bool SIGNED>
__device__ __forceinline__ void store_packed(uint8_t* __restrict__ codes, long tile, int lane, const int c[32])
{
    if constexpr (BITS == 4) {
        u32x4 q;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t wd = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) wd |= (uint32_t)c[8 * j + e] << (4 * (e / 2) + 16 * (e % 2));
            q[j] = wd;
        }
        *reinterpret_cast<u32x4*>(codes + tile * 1024 + 16 * lane) = q;
    } else if constexpr (BITS == 3) {
        uint32_t wd[3] = {0, 0, 0};
#pragma unroll
        for (int cc = 0; cc < 30; ++cc) {
            const int P = cc / 2, h = cc % 2;
            wd[P / 5] |= (uint32_t)c[cc] << (16 * h + 3 * (P % 5));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int t = 0; t < 3; ++t) wd[t] |= (((uint32_t)c[30 + h] >> t) & 1u) << (16 * h + 15);
        uint32_t* p = reinterpret_cast<uint32_t*>(codes + tile * 768 + 12 * lane);
        u32x3 q = {wd[0], wd[1], wd[2]};
        *reinterpret_cast<u32x3*>(p) = q;
    } else {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            u32x4 q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t wd = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) wd |= ((uint32_t)c[16 * p + 4 * i + b] & 0xffu) << (8 * b);
                q[i] = wd;
            }
            *reinterpret_cast<u32x4*>(codes + tile * 2048 + 1024 * p + 16 * lane) = q;
        }
    }
}

// grouped asymmetric scheme: one (row, 128 columns) group per 4 lanes
template <int BITS>
__global__ __launch_bounds__(256) void quantize_asym_kernel(const uint16_t* __restrict__ w, int K, long NT, RowWindow win,
                                                            uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                            uint16_t* __restrict__ zeros)
{
    const int KT = K / 128;
    const long tile = win.rb0 * KT * 4 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);      // ((rb * KT + kt) * 4 + t)
    if (tile >= (win.rb0 + win.n_rb) * KT * 4) return;
    const int lane = threadIdx.x & 63, t = (int)(tile & 3);
    const long rb = (tile >> 2) / KT;
    const int kt = (int)((tile >> 2) % KT);
    const long n = rb * 64 + 4 * (lane & 15) + t;
    float v[32];
    load_owned(w, K, n - 64 * win.rb0, kt, lane, v);
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) { lo = fminf(lo, v[i]); hi = fmaxf(hi, v[i]); }
    lo = fminf(lo, __shfl_xor(lo, 16)); hi = fmaxf(hi, __shfl_xor(hi, 16));
    lo = fminf(lo, __shfl_xor(lo, 32)); hi = fmaxf(hi, __shfl_xor(hi, 32));
    constexpr int QMAX = (1 << BITS) - 1;
    const float s32 = __fdiv_rn(__fsub_rn(hi, lo), (float)QMAX);
    uint16_t sh = f2h_bits(s32);
    if ((sh & 0x7fffu) == 0) sh = 0x3c00u;                 // flat group: scale 1, codes 0
    const uint16_t zh = f2h_bits(__fadd_rn(lo, 0.0f));     // min is an fp16 value; +0 makes -0 -> +0
    const float sf = h2f_bits(sh), zf = h2f_bits(zh);
    // code = rint((w - zero) / scale) with the quotient rounded to fp32 first.  The correctly rounded
    // division is ten instructions; a multiplication by a refined reciprocal is one and is off by at most
    // two units in the last place of a quotient below 256, i.e. by less than 2^-14.  So the fast quotient
    // decides the code unless it lies within 2^-13 of a half-integer, and only then (about one weight in
    // 4000, decided per element for the whole wave) is the exact division done: the codes are those of the
    // exact formula in every case.
    float rcp = __builtin_amdgcn_rcpf(sf);
    rcp = __builtin_fmaf(__builtin_fmaf(-sf, rcp, 1.0f), rcp, rcp);
    int c[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const float num = __fsub_rn(v[i], zf);
        float t = __fmul_rn(num, rcp);
        float r = __builtin_rintf(t);
        if (__builtin_amdgcn_ballot_w64(!(fabsf(__fsub_rn(t, r)) < 0.5f - 0x1p-13f)) != 0) {      // also catches NaN / Inf
            t = __fdiv_rn(num, sf);
            r = __builtin_rintf(t);
        }
        c[i] = (int)__builtin_amdgcn_fmed3f(r, 0.0f, (float)QMAX);
    }
    store_packed<BITS, false>(codes, tile, lane, c);
    if (lane < 16) {                                   // stored group-major: [K/128][N]
        const long N = NT * 16;
        scales[(long)kt * N + n] = sh;
        zeros[(long)kt * N + n] = zh;
    }
}

// per-row symmetric scheme, pass 1: scale[n] = fp16(max|w[n,:]| / 127)
__global__ __launch_bounds__(256) void row_absmax_scale_kernel(const uint16_t* __restrict__ w, int K, RowWindow win, uint16_t* __restrict__ scales)
{
    __shared__ float red[4];
    const long n = 64 * win.rb0 + blockIdx.x;
    const uint16_t* row = w + (long)blockIdx.x * K;
    float a = 0.0f;
    for (int k = threadIdx.x * 8; k < K; k += 256 * 8) {
        const h8 t = *reinterpret_cast<const h8*>(row + k);
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf((float)t[e]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        uint16_t sh = f2h_bits(__fdiv_rn(a, 127.0f));
        if ((sh & 0x7fffu) == 0) sh = 0x3c00u;
        scales[n] = sh;
    }
}

// per-row symmetric scheme, pass 2: code = clamp(rint(w / scale), -127, 127)
__global__ __launch_bounds__(256) void quantize_sym_kernel(const uint16_t* __restrict__ w, int K, RowWindow win,
                                                           uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales)
{
    const int KT = K / 128;
    const long tile = win.rb0 * KT * 4 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= (win.rb0 + win.n_rb) * KT * 4) return;
    const int lane = threadIdx.x & 63, t = (int)(tile & 3);
    const long rb = (tile >> 2) / KT;
    const int kt = (int)((tile >> 2) % KT);
    const long n = rb * 64 + 4 * (lane & 15) + t;
    float v[32];
    load_owned(w, K, n - 64 * win.rb0, kt, lane, v);
    const float sf = h2f_bits(scales[n]);
    float rcp = __builtin_amdgcn_rcpf(sf);             // guarded fast quotient, as in quantize_asym_kernel
    rcp = __builtin_fmaf(__builtin_fmaf(-sf, rcp, 1.0f), rcp, rcp);
    int c[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        float t = __fmul_rn(v[i], rcp);
        float r = __builtin_rintf(t);
        if (__builtin_amdgcn_ballot_w64(!(fabsf(__fsub_rn(t, r)) < 0.5f - 0x1p-13f)) != 0) {
            t = __fdiv_rn(v[i], sf);
            r = __builtin_rintf(t);
        }
        c[i] = (int)__builtin_amdgcn_fmed3f(r, -127.0f, 127.0f);
    }
    store_packed<8, true>(codes, tile, lane, c);
}

// 16-bit layers: the fp16 weights unchanged, reordered into tiles (piece j of a lane = operand of MFMA step j)
__global__ __launch_bounds__(256) void pack_fp16_kernel(const uint16_t* __restrict__ w, int K, RowWindow win, uint8_t* __restrict__ codes)
{
    const int KT = K / 128;
    const long tile = win.rb0 * KT * 4 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= (win.rb0 + win.n_rb) * KT * 4) return;
    const int lane = threadIdx.x & 63, t = (int)(tile & 3);
    const long rb = (tile >> 2) / KT;
    const int kt = (int)((tile >> 2) % KT);
    const long n = rb * 64 + 4 * (lane & 15) + t;
    const uint16_t* p = w + (n - 64 * win.rb0) * K + (long)kt * 128 + 8 * (lane >> 4);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        *reinterpret_cast<u32x4*>(codes + tile * 4096 + 1024 * j + 16 * lane) = *reinterpret_cast<const u32x4*>(p + 32 * j);
}

// ---- test helper: packed buffers -> fp32 weights, one code at a time from the format ----
// (kept separate from the matmul kernels' fast unpacking on purpose)
__device__ __forceinline__ int extract_code(const uint8_t* __restrict__ tile, int variant, int lane, int j, int e)
{
    if (variant == V_W4) {
        const uint32_t wd = reinterpret_cast<const uint32_t*>(tile + 16 * lane)[j];
        return (int)((wd >> (4 * (e / 2) + 16 * (e % 2))) & 15u);
    }
    if (variant == V_W3) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(tile + 12 * lane);
        const int cc = 8 * j + e, P = cc / 2, h = cc % 2;
        if (P < 15) return (int)((p[P / 5] >> (16 * h + 3 * (P % 5))) & 7u);
        int c = 0;
        for (int t = 0; t < 3; ++t) c |= (int)((p[t] >> (16 * h + 15)) & 1u) << t;
        return c;
    }
    const uint8_t b = tile[1024 * (j / 2) + 16 * lane + 8 * (j % 2) + e];
    return variant == V_I8 ? (int)(int8_t)b : (int)b;
}

__global__ __launch_bounds__(256) void unpack_dequant_kernel(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                             const uint16_t* __restrict__ zeros, int variant, int K, long NT,
                                                             float* __restrict__ out)
{
    const int KT = K / 128;
    const long tile = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= NT * KT) return;
    const int lane = threadIdx.x & 63, r = lane & 15, kq = lane >> 4, t = (int)(tile & 3);
    const long rb = (tile >> 2) / KT;
    const int kt = (int)((tile >> 2) % KT);
    const long n = rb * 64 + 4 * r + t;
    const long N = NT * 16;
    float* o = out + n * K + (long)kt * 128 + 8 * kq;
    if (variant == V_F16) {
        const uint16_t* p = reinterpret_cast<const uint16_t*>(codes + (size_t)tile * 4096);
        for (int j = 0; j < 4; ++j)
            for (int e = 0; e < 8; ++e) o[32 * j + e] = h2f_bits(p[512 * j + 8 * lane + e]);
        return;
    }
    const size_t tb = variant == V_W3 ? 768 : (variant == V_W4 ? 1024 : 2048);
    const uint8_t* tp = codes + (size_t)tile * tb;
    float s, z;
    if (variant == V_I8) { s = h2f_bits(scales[n]); z = 0.0f; }
    else { s = h2f_bits(scales[(long)kt * N + n]); z = h2f_bits(zeros[(long)kt * N + n]); }
    for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 8; ++e) {
            const float c = (float)extract_code(tp, variant, lane, j, e);
            o[32 * j + e] = __fadd_rn(__fmul_rn(s, c), z);
        }
}

}  // namespace

hipError_t launch_quantize_pack(const void* w_rows, const lpq_qdesc& d, long row0, long n_rows, const lpq_qweight& out, hipStream_t s)
{
    const long NT = d.N / 16;
    const int KT = d.K / 128;
    const RowWindow win = {row0 / 64, n_rows / 64};
    const unsigned blocks = (unsigned)(win.n_rb * KT);           // four tiles (one 64-row block step) per workgroup
    const uint16_t* wp = static_cast<const uint16_t*>(w_rows);
    uint8_t* codes = static_cast<uint8_t*>(out.codes);
    uint16_t* sc = static_cast<uint16_t*>(out.scales);
    uint16_t* zr = static_cast<uint16_t*>(out.zeros);
    if (blocks == 0) return hipSuccess;
    switch (variant_of(d)) {
    case V_W3: quantize_asym_kernel<3><<<blocks, 256, 0, s>>>(wp, d.K, NT, win, codes, sc, zr); break;
    case V_W4: quantize_asym_kernel<4><<<blocks, 256, 0, s>>>(wp, d.K, NT, win, codes, sc, zr); break;
    case V_W8: quantize_asym_kernel<8><<<blocks, 256, 0, s>>>(wp, d.K, NT, win, codes, sc, zr); break;
    case V_I8:
        row_absmax_scale_kernel<<<(unsigned)n_rows, 256, 0, s>>>(wp, d.K, win, sc);
        quantize_sym_kernel<<<blocks, 256, 0, s>>>(wp, d.K, win, codes, sc);
        break;
    case V_F16: pack_fp16_kernel<<<blocks, 256, 0, s>>>(wp, d.K, win, codes); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_unpack_dequant(const lpq_qweight& w, float* out, hipStream_t s)
{
    const long NT = w.d.N / 16;
    const long tiles = NT * (w.d.K / 128);
    unpack_dequant_kernel<<<(unsigned)((tiles + 3) / 4), 256, 0, s>>>(
        static_cast<const uint8_t*>(w.codes), static_cast<const uint16_t*>(w.scales), static_cast<const uint16_t*>(w.zeros),
        variant_of(w.d), w.d.K, NT, out);
    return hipGetLastError();
}

}  // namespace lpq
