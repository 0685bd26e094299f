// Device-side building blocks shared by the gfx950 kernels: vector types, tile loads in the
// packed storage format (see include/lpq.h), and in-register unpacking to fp16 MFMA operands.
//
// Operand convention used by every matmul kernel here (v_mfma_f32_16x16x32_f16, wave64):
//   A = activations: lane (i = lane%16 -> token, kq = lane/16) holds x[token][32*j + 8*kq + 0..7]
//   B = weights:     lane (r = lane%16 -> output row, kq)      holds w~[row][32*j + 8*kq + 0..7]
//   D (4 floats):    lane holds y[token = 4*(lane/16) + v][row = lane%16], v = 0..3
// so a lane's per-(row, group) scale and zero apply to its own B operand and to all four of
// its accumulators.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lpq {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum { SCH_FP16 = 0, SCH_ASYM = 1, SCH_SYM = 2 };
enum { GROUP = 128, TILE_ROWS = 16, BLOCK_ROWS = 64 };

// kernel-variant ids: one per (bits, scheme) the library supports
enum { V_W3 = 0, V_W4 = 1, V_W8 = 2, V_I8 = 3, V_F16 = 4, V_COUNT = 5 };

template <int V> struct VInfo;
template <> struct VInfo<V_W3>  { enum { BITS = 3,  SCHEME = SCH_ASYM, TILE_BYTES = 768 }; };
template <> struct VInfo<V_W4>  { enum { BITS = 4,  SCHEME = SCH_ASYM, TILE_BYTES = 1024 }; };
template <> struct VInfo<V_W8>  { enum { BITS = 8,  SCHEME = SCH_ASYM, TILE_BYTES = 2048 }; };
template <> struct VInfo<V_I8>  { enum { BITS = 8,  SCHEME = SCH_SYM,  TILE_BYTES = 2048 }; };
template <> struct VInfo<V_F16> { enum { BITS = 16, SCHEME = SCH_FP16, TILE_BYTES = 4096 }; };

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ h2 splat(_Float16 v) { h2 r = {v, v}; return r; }
__device__ __forceinline__ h2 pk_fma(h2 a, h2 b, h2 c) { return __builtin_elementwise_fma(a, b, c); }

// ---- packed codes of one 16x128 tile, as held by one lane ------------------------------
template <int V> struct WRaw;
template <> struct WRaw<V_W3>  { u32x3 q; };
template <> struct WRaw<V_W4>  { u32x4 q; };
template <> struct WRaw<V_W8>  { u32x4 q[2]; };
template <> struct WRaw<V_I8>  { u32x4 q[2]; };
template <> struct WRaw<V_F16> { u32x4 q[4]; };

// codes: base of the packed buffer.  A 64-row x 128-column block (rb, kt) holds four tiles back
// to back; tile t has rows 64*rb + 4*r + t.  One wave that owns the block reads 4 * TILE_BYTES
// contiguous bytes per 128-column step, and consecutive steps are contiguous too.
template <int V>
__device__ __forceinline__ WRaw<V> load_tile(const uint8_t* __restrict__ codes, long rb, int KT, int kt, int t, int lane)
{
    WRaw<V> w;
    const uint8_t* tile = codes + (((size_t)rb * KT + kt) * 4 + t) * (size_t)VInfo<V>::TILE_BYTES;
    if constexpr (V == V_W3) {
        w.q = __builtin_nontemporal_load(reinterpret_cast<const u32x3*>(tile + 12 * lane));
    } else if constexpr (V == V_W4) {
        w.q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 16 * lane));
    } else if constexpr (V == V_W8 || V == V_I8) {
        w.q[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 16 * lane));
        w.q[1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 1024 + 16 * lane));
    } else {   // fp16 weights: piece j is the operand of MFMA step j as it stands
#pragma unroll
        for (int j = 0; j < 4; ++j) w.q[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + 1024 * j + 16 * lane));
    }
    return w;
}

// The same loads from the lane's own address in the tile (tile start + 12 or 16 bytes per lane).
template <int V>
__device__ __forceinline__ WRaw<V> load_tile_at(const uint8_t* __restrict__ p)
{
    WRaw<V> w;
    if constexpr (V == V_W3) {
        w.q = __builtin_nontemporal_load(reinterpret_cast<const u32x3*>(p));
    } else if constexpr (V == V_W4) {
        w.q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    } else if constexpr (V == V_W8 || V == V_I8) {
        w.q[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        w.q[1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + 1024));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) w.q[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + 1024 * j));
    }
    return w;
}

// Output epilogue: activation (lpq_activation) on acc + bias, in fp32.
__device__ __forceinline__ float apply_activation(float v, int act)
{
    if (act == LPQ_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == LPQ_ACT_GELU_TANH) return 0.5f * v * (1.0f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
    return v;
}

// ---- unpack to fp16 values that are exactly the integer codes --------------------------
// OR-ing a code field into the mantissa of fp16 1024.0 (0x6400) gives 1024 + c*code exactly,
// c = 2^(field's bit offset in the half-word); one packed op then removes the offset.

__device__ __forceinline__ h2 magic_to_int(uint32_t biased, int log2c)
{
    // (1024 + c*q) -> q, exact: q <= 255 is an fp16 integer
    if (log2c == 0) return as_h2(biased) - splat((_Float16)1024.0f);
    const _Float16 inv = (_Float16)(1.0f / (float)(1 << log2c));
    const _Float16 off = (_Float16)(-1024.0f / (float)(1 << log2c));
    return pk_fma(as_h2(biased), splat(inv), splat(off));
}

// (x & mask) | magic in one VALU op.  The compiler splits this into v_and + v_or when both constants
// are literals; with the mask in an SGPR and the magic in a VGPR it is a single v_and_or_b32.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic_vgpr)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(magic_vgpr));
    return r;
}

// out[j] = the lane's 8 operand values of MFMA step j, as integer-valued fp16 codes
template <int V>
__device__ __forceinline__ void unpack_codes(const WRaw<V>& w, h8 out[4])
{
    constexpr uint32_t MAGIC = 0x64006400u;
    uint32_t magic_v;                                   // the magic constant held in a VGPR (see and_or)
    asm("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(MAGIC));
    if constexpr (V == V_W4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t q = w.q[j], t = q >> 8;
            h2 p0 = magic_to_int(and_or(q, 0x000F000Fu, magic_v), 0);
            h2 p1 = magic_to_int(and_or(q, 0x00F000F0u, magic_v), 4);
            h2 p2 = magic_to_int(and_or(t, 0x000F000Fu, magic_v), 0);
            h2 p3 = magic_to_int(and_or(t, 0x00F000F0u, magic_v), 4);
            h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
            out[j] = o;
        }
    } else if constexpr (V == V_W3) {
        h2 pr[16];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t q = w.q[i], t = q >> 9;
            pr[5 * i + 0] = magic_to_int(and_or(q, 0x00070007u, magic_v), 0);
            pr[5 * i + 1] = magic_to_int(and_or(q, 0x00380038u, magic_v), 3);
            pr[5 * i + 2] = magic_to_int(and_or(q, 0x01C001C0u, magic_v), 6);
            pr[5 * i + 3] = magic_to_int(and_or(t, 0x00070007u, magic_v), 0);
            pr[5 * i + 4] = magic_to_int(and_or(t, 0x00380038u, magic_v), 3);
        }
        uint32_t u = and_or(w.q[0] >> 15, 0x00010001u, magic_v);
        u = and_or(w.q[1] >> 14, 0x00020002u, u);
        u = and_or(w.q[2] >> 13, 0x00040004u, u);
        pr[15] = magic_to_int(u, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            h8 o = {pr[4 * j][0], pr[4 * j][1], pr[4 * j + 1][0], pr[4 * j + 1][1],
                    pr[4 * j + 2][0], pr[4 * j + 2][1], pr[4 * j + 3][0], pr[4 * j + 3][1]};
            out[j] = o;
        }
    } else if constexpr (V == V_W8 || V == V_I8) {
        constexpr uint32_t M8 = 0x64646464u;
        const _Float16 off = (V == V_I8) ? (_Float16)1152.0f : (_Float16)1024.0f;   // 1024 (+128 for signed)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t a = w.q[j >> 1][2 * (j & 1)], b = w.q[j >> 1][2 * (j & 1) + 1];
            if constexpr (V == V_I8) { a ^= 0x80808080u; b ^= 0x80808080u; }       // two's complement -> offset binary
            h2 p0 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00050004u)) - splat(off);
            h2 p1 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00070006u)) - splat(off);
            h2 p2 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00050004u)) - splat(off);
            h2 p3 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00070006u)) - splat(off);
            h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
            out[j] = o;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = __builtin_bit_cast(h8, w.q[j]);
    }
}

// ---- unpack to fp16 SUBNORMALS whose value is code * 2^-24 ------------------------------
// A code field moved to mantissa bits 0.. of a half-word with a zero exponent IS the fp16
// subnormal code * 2^-24, so one AND per pair of codes yields an MFMA operand (the matrix cores
// take fp16 subnormals at full precision).  The factor 2^24 is folded into the group scale, which
// is applied in fp32 after the 128-column partial product.  Signed 8-bit codes come out offset by
// +128 (two's complement with the top bit flipped); the caller removes 128 * sum(x).
// One MFMA step (32 columns: j) of the codes as subnormals; callers interleave the unpacking of
// step j + 1 with the matrix instructions of step j.
template <int V>
__device__ __forceinline__ h8 unpack_subnormal_step(const WRaw<V>& w, int j)
{
    if constexpr (V == V_W4) {
        constexpr uint32_t M4 = 0x000F000Fu;
        const uint32_t q = w.q[j];
        // the top nibble of each half-word needs no mask: a packed 16-bit shift fills each half with zeros on its own
        typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
        const u16x2 top = __builtin_bit_cast(u16x2, q) >> (uint16_t)12;
        const u32x4 o = {q & M4, (q >> 4) & M4, (q >> 8) & M4, __builtin_bit_cast(uint32_t, top)};
        return __builtin_bit_cast(h8, o);
    } else if constexpr (V == V_W3) {
        constexpr uint32_t M3 = 0x00070007u;
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int P = 4 * j + k;
            if (P < 15) o[k] = (w.q[P / 5] >> (3 * (P % 5))) & M3;
            else o[k] = ((w.q[0] >> 15) & 0x00010001u) | ((w.q[1] >> 14) & 0x00020002u) | ((w.q[2] >> 13) & 0x00040004u);
        }
        return __builtin_bit_cast(h8, o);
    } else if constexpr (V == V_W8 || V == V_I8) {
        uint32_t a = w.q[j >> 1][2 * (j & 1)], b = w.q[j >> 1][2 * (j & 1) + 1];
        if constexpr (V == V_I8) { a ^= 0x80808080u; b ^= 0x80808080u; }
        const u32x4 o = {__builtin_amdgcn_perm(a, 0u, 0x0c050c04u), __builtin_amdgcn_perm(a, 0u, 0x0c070c06u),
                         __builtin_amdgcn_perm(b, 0u, 0x0c050c04u), __builtin_amdgcn_perm(b, 0u, 0x0c070c06u)};
        return __builtin_bit_cast(h8, o);
    } else {
        return __builtin_bit_cast(h8, w.q[j]);
    }
}

// ---- 3-bit codes as subnormals WHERE THEY LIE ---------------------------------------------
// A field need not be moved to bit 0 to be an operand: masked in place at bit offset s <= 6 (so that it ends below
// the exponent's second bit) the half-word is the fp16 number code * 2^s * 2^-24, exactly.  The factor 2^s is taken out
// on the other side of the product: the activations of those columns are multiplied by 2^-s beforehand (an exact
// scaling, together with a power of two per token row that keeps every element in the normal range; the kernel that
// prepares a decode launch's activations does it).  A 3-bit half-word then needs one shift (by 9, for its fields 3
// and 4) instead of four.  inplace_class<V>(j, k) is the power of 8 that output register k of MFMA step j carries:
// columns 2k and 2k + 1 of the lane's eight.
template <int V> __device__ __host__ constexpr int inplace_class(int j, int k)
{
    static_assert(V == V_W3, "only 3-bit codes are read in place");
    return (4 * j + k) < 15 ? ((4 * j + k) % 5) % 3 : 0;
}

template <int V>
__device__ __forceinline__ h8 unpack_inplace_step(const WRaw<V>& w, int j)
{
    static_assert(V == V_W3, "only 3-bit codes are read in place");
    u32x4 o;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int P = 4 * j + k;
        if (P < 15) {
            const int f = P % 5;
            const uint32_t src = f >= 3 ? (w.q[P / 5] >> 9) : w.q[P / 5];
            o[k] = src & (0x00070007u << (3 * (f % 3)));
        } else {
            o[k] = ((w.q[0] >> 15) & 0x00010001u) | ((w.q[1] >> 14) & 0x00020002u) | ((w.q[2] >> 13) & 0x00040004u);
        }
    }
    return __builtin_bit_cast(h8, o);
}

// One MFMA step (32 columns: j) of a tile as integer-valued fp16 codes (the 0x6400 mantissa trick above).
template <int V>
__device__ __forceinline__ h8 unpack_codes_step(const WRaw<V>& w, int j)
{
    constexpr uint32_t MAGIC = 0x64006400u;
    uint32_t magic_v;
    asm("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(MAGIC));
    if constexpr (V == V_W4) {
        const uint32_t q = w.q[j], t = q >> 8;
        const h2 p0 = magic_to_int(and_or(q, 0x000F000Fu, magic_v), 0);
        const h2 p1 = magic_to_int(and_or(q, 0x00F000F0u, magic_v), 4);
        const h2 p2 = magic_to_int(and_or(t, 0x000F000Fu, magic_v), 0);
        const h2 p3 = magic_to_int(and_or(t, 0x00F000F0u, magic_v), 4);
        const h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
        return o;
    } else if constexpr (V == V_W3) {
        h2 pr[4];                                   // pairs P = 4*j .. 4*j + 3
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int P = 4 * j + k;
            if (P < 15) {
                const int i = P / 5, f = P % 5, ff = f % 3;        // fields 3, 4 sit at bits 9, 12: shift them down first
                const uint32_t src = (f >= 3) ? (w.q[i] >> 9) : w.q[i];
                pr[k] = magic_to_int(and_or(src, 0x00070007u << (3 * ff), magic_v), 3 * ff);
            } else {
                uint32_t u = and_or(w.q[0] >> 15, 0x00010001u, magic_v);
                u = and_or(w.q[1] >> 14, 0x00020002u, u);
                u = and_or(w.q[2] >> 13, 0x00040004u, u);
                pr[k] = magic_to_int(u, 0);
            }
        }
        const h8 o = {pr[0][0], pr[0][1], pr[1][0], pr[1][1], pr[2][0], pr[2][1], pr[3][0], pr[3][1]};
        return o;
    } else if constexpr (V == V_W8 || V == V_I8) {
        constexpr uint32_t M8 = 0x64646464u;
        const _Float16 off = (V == V_I8) ? (_Float16)1152.0f : (_Float16)1024.0f;   // 1024 (+128 for signed)
        uint32_t a = w.q[j >> 1][2 * (j & 1)], b = w.q[j >> 1][2 * (j & 1) + 1];
        if constexpr (V == V_I8) { a ^= 0x80808080u; b ^= 0x80808080u; }           // two's complement -> offset binary
        const h2 p0 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00050004u)) - splat(off);
        const h2 p1 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00070006u)) - splat(off);
        const h2 p2 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00050004u)) - splat(off);
        const h2 p3 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00070006u)) - splat(off);
        const h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
        return o;
    } else {
        return __builtin_bit_cast(h8, w.q[j]);
    }
}

// The same for two MFMA steps only (j = 2*half, 2*half + 1): the compute-bound kernels build their
// operands half a 128-column step at a time to keep 32 instead of 64 operand registers live.
// `piece8`: for the 8-bit variants, which of w.q[] holds the 16-byte piece of this half (callers that
// load one piece at a time keep it in q[0]).
template <int V>
__device__ __forceinline__ void unpack_codes_half(const WRaw<V>& w, int half, h8 out[2], int piece8 = -1)
{
    constexpr uint32_t MAGIC = 0x64006400u;
    uint32_t magic_v;
    asm("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(MAGIC));
    if constexpr (V == V_W4) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const uint32_t q = w.q[2 * half + jj], t = q >> 8;
            h2 p0 = magic_to_int(and_or(q, 0x000F000Fu, magic_v), 0);
            h2 p1 = magic_to_int(and_or(q, 0x00F000F0u, magic_v), 4);
            h2 p2 = magic_to_int(and_or(t, 0x000F000Fu, magic_v), 0);
            h2 p3 = magic_to_int(and_or(t, 0x00F000F0u, magic_v), 4);
            h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
            out[jj] = o;
        }
    } else if constexpr (V == V_W3) {
        h2 pr[8];                                   // pairs P = 8*half .. 8*half + 7
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int P = 8 * half + k;
            if (P < 15) {
                const int i = P / 5, f = P % 5, ff = f % 3;        // fields 3, 4 sit at bits 9, 12: shift them down first
                const uint32_t src = (f >= 3) ? (w.q[i] >> 9) : w.q[i];
                pr[k] = magic_to_int(and_or(src, 0x00070007u << (3 * ff), magic_v), 3 * ff);
            } else {
                uint32_t u = and_or(w.q[0] >> 15, 0x00010001u, magic_v);
                u = and_or(w.q[1] >> 14, 0x00020002u, u);
                u = and_or(w.q[2] >> 13, 0x00040004u, u);
                pr[k] = magic_to_int(u, 0);
            }
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            h8 o = {pr[4 * jj][0], pr[4 * jj][1], pr[4 * jj + 1][0], pr[4 * jj + 1][1],
                    pr[4 * jj + 2][0], pr[4 * jj + 2][1], pr[4 * jj + 3][0], pr[4 * jj + 3][1]};
            out[jj] = o;
        }
    } else if constexpr (V == V_W8 || V == V_I8) {
        constexpr uint32_t M8 = 0x64646464u;
        const _Float16 off = (V == V_I8) ? (_Float16)1152.0f : (_Float16)1024.0f;   // 1024 (+128 for signed)
        const u32x4 piece = w.q[piece8 < 0 ? half : piece8];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            uint32_t a = piece[2 * jj], b = piece[2 * jj + 1];
            if constexpr (V == V_I8) { a ^= 0x80808080u; b ^= 0x80808080u; }
            h2 p0 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00050004u)) - splat(off);
            h2 p1 = as_h2(__builtin_amdgcn_perm(a, M8, 0x00070006u)) - splat(off);
            h2 p2 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00050004u)) - splat(off);
            h2 p3 = as_h2(__builtin_amdgcn_perm(b, M8, 0x00070006u)) - splat(off);
            h8 o = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
            out[jj] = o;
        }
    } else {
        out[0] = __builtin_bit_cast(h8, w.q[2 * half]);
        out[1] = __builtin_bit_cast(h8, w.q[2 * half + 1]);
    }
}

// One pair of a lane's 32 codes (pair P = 0 .. 15: columns 2 P % 8, 2 P % 8 + 1 of the lane's eight in MFMA step P / 4)
// as integer-valued fp16, 3- and 4-bit codes: what unpack_codes_half yields, one register at a time, for callers that
// spread the unpacking thinly between matrix instructions.
template <int V>
__device__ __forceinline__ h2 unpack_codes_pair(const WRaw<V>& w, int P)
{
    static_assert(V == V_W3 || V == V_W4, "3- and 4-bit codes");
    constexpr uint32_t MAGIC = 0x64006400u;
    uint32_t magic_v;
    asm("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(MAGIC));
    if constexpr (V == V_W4) {
        const uint32_t q = w.q[P / 4], src = (P % 4) >= 2 ? q >> 8 : q;
        return (P % 2) ? magic_to_int(and_or(src, 0x00F000F0u, magic_v), 4) : magic_to_int(and_or(src, 0x000F000Fu, magic_v), 0);
    } else {
        if (P < 15) {
            const int i = P / 5, f = P % 5, ff = f % 3;            // fields 3, 4 sit at bits 9, 12: shift them down first
            const uint32_t src = (f >= 3) ? (w.q[i] >> 9) : w.q[i];
            return magic_to_int(and_or(src, 0x00070007u << (3 * ff), magic_v), 3 * ff);
        }
        uint32_t u = and_or(w.q[0] >> 15, 0x00010001u, magic_v);
        u = and_or(w.q[1] >> 14, 0x00020002u, u);
        u = and_or(w.q[2] >> 13, 0x00040004u, u);
        return magic_to_int(u, 0);
    }
}

// w~ = scale * code + zero for the two operands of a half step
__device__ __forceinline__ void apply_scale_zero_half(h8 v[2], _Float16 s, _Float16 z)
{
    const h8 s8 = {s, s, s, s, s, s, s, s}, z8 = {z, z, z, z, z, z, z, z};
    v[0] = __builtin_elementwise_fma(v[0], s8, z8);
    v[1] = __builtin_elementwise_fma(v[1], s8, z8);
}

// w~ = scale * code + zero with one fp16 rounding per weight (packed fma)
__device__ __forceinline__ void apply_scale_zero(h8 v[4], _Float16 s, _Float16 z)
{
    const h8 s8 = {s, s, s, s, s, s, s, s}, z8 = {z, z, z, z, z, z, z, z};
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = __builtin_elementwise_fma(v[j], s8, z8);
}

__device__ __forceinline__ f4 mfma16(h8 a, h8 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }

// 32x32x16 does twice the multiply-accumulates of 16x16x32 per operand register read (and per LDS operand read), at the
// same rate per cycle (counters: 32 against 16-18 matrix-pipe cycles per instruction), so the compute-bound kernels
// use it.  Its B operand wants lane = row % 32 + 32 * (k half); two tiles in
// the 16x16x32 layout (lane = row % 16 + 16 * kq) become two such operands with one
// v_permlane16_swap per register: afterwards `lo` holds {tile a kq0, tile b kq0, tile a kq2, tile b kq2}
// and `hi` holds {tile a kq1, tile b kq1, tile a kq3, tile b kq3}, i.e. 32 rows x (k slots kq, kq+2).
typedef float f16x __attribute__((ext_vector_type(16)));
__device__ __forceinline__ f16x mfma32(h8 a, h8 b, f16x c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ void pair_tiles_for_mfma32(h8& a, h8& b)
{
    u32x4 ua = __builtin_bit_cast(u32x4, a), ub = __builtin_bit_cast(u32x4, b);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const u32x2 s = __builtin_amdgcn_permlane16_swap(ua[i], ub[i], false, false);
        ua[i] = s[0];
        ub[i] = s[1];
    }
    a = __builtin_bit_cast(h8, ua);
    b = __builtin_bit_cast(h8, ub);
}

}  // namespace lpq
