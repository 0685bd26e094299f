/*
 * lpq_oracle.c -- plain, slow CPU oracle for the mixed-precision quantized-linear path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its Python
 * binding) may include, link, import or call this file; it exists so that the GPU kernels
 * can be checked element by element against an implementation that is easy to compare with
 * the paper by eye.  It shares no code, header, table or constant with the HIP sources.
 *
 * What it computes (LLM-PQ, arXiv 2403.01136):
 *   - Sec. 2.4 "Quantization in LLM": code = round((x - q_x) / s_x),
 *     s_x = (x_max - x_min) / (2^b - 1), dequantised value = s_x * code + q_x.
 *     q_x is read as the minimum of the vector (a floating offset), the vector as one
 *     (output row, 128 consecutive input channels) group.
 *   - Sec. 4.2, scaling-factor definitions below Theorem 1: the asymmetric form above and
 *     the symmetric form S = max(|W_max|, |W_min|) / (2^(b-1) - 1), used here for the
 *     per-output-row signed 8-bit scheme.
 *   - Sec. 4.1 "Weight Storage": a quantised linear holds (#weights) * bit / 8 bytes, so
 *     the packed codes are dense (3-bit codes are not padded to 4).
 *   - Sec. 4.3 (BITs = {3, 4, 8, 16}): 16 means the FP16 weights are used unchanged.
 *   - App. A.1 (deterministic rounding): |w - dequant(w)| <= s_w / 2.
 *
 * Steps, in the order the paper gives them:
 *   O1 group statistics (min, max | row absmax), fp32
 *   O2 scale = fp16(range / (2^b - 1)), zero = fp16(min)
 *   O3 code = clamp(rint((w - zero) / scale)), then bit-packing per the storage format
 *   O4 dequantise in fp32: scale * code + zero
 *   O5 y = x . w~^T accumulated in fp64
 *
 * fp32 arithmetic is IEEE round-to-nearest-even with no fused contraction (build with
 * -ffp-contract=off, no fast-math).  fp16 <-> fp32 conversions are written out below.
 *
 * Storage format of the packed buffers (a convention of this project, restated here from its
 * prose description, not shared with the GPU sources):
 *   W is [N][K], K contiguous; N % 64 == 0, K % 128 == 0.  A block is 64 rows x 128 columns;
 *   blocks are stored in order (n/64) * (K/128) + k/128.  A block holds four tiles one after
 *   the other; tile t holds the 16 rows 64*(n/64) + 4*r + t (r = 0..15), i.e. t = n % 4 and
 *   r = (n % 64) / 4.  A tile is owned by 64 "lanes", lane = 16 * kq + r (kq = 0..3); the lane
 *   owns the 32 codes of its row at block columns 32*j + 8*kq + e (j = 0..3, e = 0..7),
 *   numbered c = 8*j + e.
 *     4-bit: 1024-byte tile; 16 bytes per lane at 16*lane: four LE u32, word j; code e sits at
 *            bit 4*(e/2) + 16*(e%2) of word j.
 *     3-bit: 768-byte tile; 12 bytes per lane at 12*lane: three LE u32.  Pair P = c/2, half
 *            h = c%2.  P < 15: word P/5, bits 16*h + 3*(P%5) .. +2.  P == 15: bit i of the code
 *            is bit 16*h + 15 of word i (i = 0, 1, 2).
 *     8-bit: 2048-byte tile; 32 bytes per lane in two 16-byte pieces: piece p (j = 2p, 2p+1) at
 *            1024*p + 16*lane; byte 8*(j%2) + e holds code (j, e).  Signed codes are two's
 *            complement.
 *     16-bit: 4096-byte tile of unchanged fp16 weights; 64 bytes per lane as four 16-byte pieces:
 *            piece j at 1024*j + 16*lane, element e (2 bytes, little-endian) at byte 2*e.
 *   scales (and zeros) as stored: fp16 [K/128][N] (group-major: index g*N + n); per-row
 *   scheme: scales fp16 [N], no zeros.  lpq_oracle_quantize returns them in the natural
 *   [N][K/128] order; lpq_oracle_store_scales rearranges them into the stored order.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#pragma STDC FP_CONTRACT OFF

enum { ORC_FP16 = 0, ORC_ASYM_GROUP = 1, ORC_SYM_CHANNEL = 2 };
enum { ORC_GROUP = 128, ORC_BLOCK_ROWS = 64 };

/* ---- fp16 <-> fp32, written out ------------------------------------------------------ */

/* Exact: every fp16 value is an fp32 value. */
float lpq_oracle_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t  e    = (h >> 10) & 0x1f;
    uint32_t m    = h & 0x3ffu;
    double v;
    if (e == 0)       v = ldexp((double)m, -24);              /* zero / subnormal */
    else if (e == 31) v = m ? (double)NAN : (double)INFINITY;
    else              v = ldexp((double)(m + 1024u), e - 25);
    return (float)(sign ? -v : v);
}

/* fp32 -> fp16, round to nearest, ties to even; overflow -> inf; subnormals produced. */
uint16_t lpq_oracle_f2h(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) return (uint16_t)(sign | 0x7c00u | ((a > 0x7f800000u) ? 0x200u : 0u));
    double v = fabs((double)f);
    if (v == 0.0) return sign;
    int ex; (void)frexp(v, &ex);           /* v = frac * 2^ex, frac in [0.5, 1) */
    int e = ex - 1;                        /* v in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;                  /* subnormal range: fixed quantum 2^-24 */
    double q = ldexp(v, 10 - e);           /* in units of the fp16 quantum at this exponent */
    double r = nearbyint(q);               /* default rounding mode: nearest, ties to even */
    if (r >= 2048.0) { r *= 0.5; e += 1; }
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    if (r < 1024.0) return (uint16_t)(sign | (uint16_t)r);                 /* subnormal */
    return (uint16_t)(sign | ((uint32_t)(e + 15) << 10) | ((uint32_t)r - 1024u));
}

/* ---- sizes (Sec. 4.1: bytes = weights * bit / 8) ------------------------------------- */

static int check_desc(int bits, int scheme, long K, long N)
{
    if (K <= 0 || N <= 0 || K % ORC_GROUP || N % ORC_BLOCK_ROWS) return -1;
    if (scheme == ORC_FP16)        return bits == 16 ? 0 : -1;
    if (scheme == ORC_ASYM_GROUP)  return (bits == 3 || bits == 4 || bits == 8) ? 0 : -1;
    if (scheme == ORC_SYM_CHANNEL) return bits == 8 ? 0 : -1;
    return -1;
}

int lpq_oracle_packed_sizes(int bits, int scheme, long K, long N,
                            size_t *code_bytes, size_t *scale_bytes, size_t *zero_bytes)
{
    if (check_desc(bits, scheme, K, N)) return -1;
    *code_bytes = (size_t)K * (size_t)N * (size_t)bits / 8u;
    if (scheme == ORC_ASYM_GROUP)       { *scale_bytes = (size_t)N * (size_t)(K / ORC_GROUP) * 2u; *zero_bytes = *scale_bytes; }
    else if (scheme == ORC_SYM_CHANNEL) { *scale_bytes = (size_t)N * 2u; *zero_bytes = 0; }
    else                                { *scale_bytes = 0; *zero_bytes = 0; }
    return 0;
}

/* ---- O1-O3: round-to-nearest quantiser ----------------------------------------------- */

/* codes: int32 [N][K] (signed for the per-row scheme); scales/zeros: fp16 bit patterns. */
int lpq_oracle_quantize(const uint16_t *w, int bits, int scheme, long K, long N,
                        int32_t *codes, uint16_t *scales, uint16_t *zeros)
{
    if (check_desc(bits, scheme, K, N) || scheme == ORC_FP16) return -1;
    const long G = K / ORC_GROUP;
    if (scheme == ORC_ASYM_GROUP) {
        const int   qmax  = (1 << bits) - 1;
        const float fqmax = (float)qmax;
        #pragma omp parallel for schedule(static)
        for (long n = 0; n < N; ++n) {
            for (long g = 0; g < G; ++g) {
                const uint16_t *wg = w + n * K + g * ORC_GROUP;
                /* O1: group minimum and maximum */
                float lo = lpq_oracle_h2f(wg[0]), hi = lo;
                for (int k = 1; k < ORC_GROUP; ++k) {
                    float v = lpq_oracle_h2f(wg[k]);
                    if (v < lo) lo = v;
                    if (v > hi) hi = v;
                }
                /* O2: s = (max - min) / (2^b - 1), kept in fp16; zero-point = min (an fp16
                 * value already; "+ 0" only turns -0 into +0 so the stored bits are unique) */
                volatile float range = hi - lo;
                volatile float s32   = range / fqmax;
                uint16_t sh = lpq_oracle_f2h(s32);
                if ((sh & 0x7fffu) == 0) sh = 0x3c00u;       /* flat group: scale 1, codes 0 */
                uint16_t zh = lpq_oracle_f2h(lo + 0.0f);
                scales[n * G + g] = sh;
                zeros[n * G + g]  = zh;
                /* O3: code = round((w - zero) / scale), with the stored fp16 scale */
                const float sf = lpq_oracle_h2f(sh), zf = lpq_oracle_h2f(zh);
                for (int k = 0; k < ORC_GROUP; ++k) {
                    volatile float d = lpq_oracle_h2f(wg[k]) - zf;
                    volatile float t = d / sf;
                    float r = nearbyintf(t);
                    int c = (r < 0.0f) ? 0 : (r > fqmax ? qmax : (int)r);
                    codes[n * K + g * ORC_GROUP + k] = c;
                }
            }
        }
    } else { /* ORC_SYM_CHANNEL: S = max|w| / (2^(b-1) - 1) per output row */
        #pragma omp parallel for schedule(static)
        for (long n = 0; n < N; ++n) {
            float a = 0.0f;
            for (long k = 0; k < K; ++k) {
                float v = fabsf(lpq_oracle_h2f(w[n * K + k]));
                if (v > a) a = v;
            }
            volatile float s32 = a / 127.0f;
            uint16_t sh = lpq_oracle_f2h(s32);
            if ((sh & 0x7fffu) == 0) sh = 0x3c00u;
            scales[n] = sh;
            const float sf = lpq_oracle_h2f(sh);
            for (long k = 0; k < K; ++k) {
                volatile float t = lpq_oracle_h2f(w[n * K + k]) / sf;
                float r = nearbyintf(t);
                int c = (r < -127.0f) ? -127 : (r > 127.0f ? 127 : (int)r);
                codes[n * K + k] = c;
            }
        }
    }
    return 0;
}

/* ---- O3 (second half): bit-packing --------------------------------------------------- */

static void put_bits_le32(uint8_t *base, int word, int bit, unsigned nbits, uint32_t value)
{
    /* OR `value` (nbits wide) into little-endian 32-bit word `word` at bit offset `bit` */
    for (unsigned i = 0; i < nbits; ++i) {
        if ((value >> i) & 1u) {
            int b = bit + (int)i;
            base[4 * word + b / 8] |= (uint8_t)(1u << (b % 8));
        }
    }
}

static uint32_t get_bits_le32(const uint8_t *base, int word, int bit, unsigned nbits)
{
    uint32_t v = 0;
    for (unsigned i = 0; i < nbits; ++i) {
        int b = bit + (int)i;
        if ((base[4 * word + b / 8] >> (b % 8)) & 1u) v |= 1u << i;
    }
    return v;
}

/* Where code (n, k) lives: byte offset of its tile, then lane, j, e inside the tile. */
static size_t locate(long n, long k, long K, int bits, int *lane, int *j, int *e)
{
    const long KT = K / ORC_GROUP;
    const size_t tile_bytes = (size_t)16 * ORC_GROUP * (size_t)bits / 8u;
    const long block = n / ORC_BLOCK_ROWS, kt = k / ORC_GROUP;
    const int  t = (int)(n % 4), r = (int)((n % ORC_BLOCK_ROWS) / 4);
    const int  kk = (int)(k % ORC_GROUP);
    *j = kk / 32;
    *e = kk % 8;
    *lane = 16 * ((kk % 32) / 8) + r;
    return (((size_t)block * (size_t)KT + (size_t)kt) * 4u + (size_t)t) * tile_bytes;
}

int lpq_oracle_pack(const int32_t *codes, int bits, int scheme, long K, long N, uint8_t *packed)
{
    if (check_desc(bits, scheme, K, N) || scheme == ORC_FP16) return -1;
    memset(packed, 0, (size_t)K * (size_t)N * (size_t)bits / 8u);
    for (long n = 0; n < N; ++n) {
        for (long k = 0; k < K; ++k) {
            int lane, j, e;
            uint8_t *tile = packed + locate(n, k, K, bits, &lane, &j, &e);
            int32_t c = codes[n * K + k];
            if (bits == 4) {
                if (c < 0 || c > 15) return -2;
                put_bits_le32(tile + 16 * lane, j, 4 * (e / 2) + 16 * (e % 2), 4, (uint32_t)c);
            } else if (bits == 3) {
                if (c < 0 || c > 7) return -2;
                int cc = 8 * j + e, P = cc / 2, h = cc % 2;
                if (P < 15) put_bits_le32(tile + 12 * lane, P / 5, 16 * h + 3 * (P % 5), 3, (uint32_t)c);
                else for (int t = 0; t < 3; ++t) put_bits_le32(tile + 12 * lane, t, 16 * h + 15, 1, ((uint32_t)c >> t) & 1u);
            } else { /* 8 */
                if (scheme == ORC_ASYM_GROUP ? (c < 0 || c > 255) : (c < -127 || c > 127)) return -2;
                tile[1024 * (j / 2) + 16 * lane + 8 * (j % 2) + e] = (uint8_t)(c & 0xff);
            }
        }
    }
    return 0;
}

int lpq_oracle_unpack(const uint8_t *packed, int bits, int scheme, long K, long N, int32_t *codes)
{
    if (check_desc(bits, scheme, K, N) || scheme == ORC_FP16) return -1;
    for (long n = 0; n < N; ++n) {
        for (long k = 0; k < K; ++k) {
            int lane, j, e;
            const uint8_t *tile = packed + locate(n, k, K, bits, &lane, &j, &e);
            int32_t c;
            if (bits == 4) {
                c = (int32_t)get_bits_le32(tile + 16 * lane, j, 4 * (e / 2) + 16 * (e % 2), 4);
            } else if (bits == 3) {
                int cc = 8 * j + e, P = cc / 2, h = cc % 2;
                if (P < 15) c = (int32_t)get_bits_le32(tile + 12 * lane, P / 5, 16 * h + 3 * (P % 5), 3);
                else { c = 0; for (int t = 0; t < 3; ++t) c |= (int32_t)get_bits_le32(tile + 12 * lane, t, 16 * h + 15, 1) << t; }
            } else {
                uint8_t b = tile[1024 * (j / 2) + 16 * lane + 8 * (j % 2) + e];
                c = (scheme == ORC_SYM_CHANNEL) ? (int32_t)(int8_t)b : (int32_t)b;
            }
            codes[n * K + k] = c;
        }
    }
    return 0;
}

/* 16-bit layers: the fp16 weights are stored unchanged, but in the same tile order. */
int lpq_oracle_pack_fp16(const uint16_t *w, long K, long N, uint8_t *packed)
{
    if (check_desc(16, ORC_FP16, K, N)) return -1;
    for (long n = 0; n < N; ++n) {
        for (long k = 0; k < K; ++k) {
            int lane, j, e;
            uint8_t *tile = packed + locate(n, k, K, 16, &lane, &j, &e);
            uint16_t v = w[n * K + k];
            tile[1024 * j + 16 * lane + 2 * e]     = (uint8_t)(v & 0xffu);
            tile[1024 * j + 16 * lane + 2 * e + 1] = (uint8_t)(v >> 8);
        }
    }
    return 0;
}

int lpq_oracle_unpack_fp16(const uint8_t *packed, long K, long N, uint16_t *w)
{
    if (check_desc(16, ORC_FP16, K, N)) return -1;
    for (long n = 0; n < N; ++n) {
        for (long k = 0; k < K; ++k) {
            int lane, j, e;
            const uint8_t *tile = packed + locate(n, k, K, 16, &lane, &j, &e);
            w[n * K + k] = (uint16_t)(tile[1024 * j + 16 * lane + 2 * e] | (tile[1024 * j + 16 * lane + 2 * e + 1] << 8));
        }
    }
    return 0;
}

/* Natural [N][K/128] order -> stored [K/128][N] order (grouped scheme only). */
int lpq_oracle_store_scales(const uint16_t *natural, long K, long N, uint16_t *stored)
{
    if (K <= 0 || N <= 0 || K % ORC_GROUP) return -1;
    const long G = K / ORC_GROUP;
    for (long n = 0; n < N; ++n)
        for (long g = 0; g < G; ++g) stored[g * N + n] = natural[n * G + g];
    return 0;
}

/* ---- O4: dequantise in fp32 (Sec. 2.4: x~ = s * code + q) ----------------------------- */

int lpq_oracle_dequant(const int32_t *codes, const uint16_t *scales, const uint16_t *zeros,
                       int bits, int scheme, long K, long N, float *w_deq)
{
    if (check_desc(bits, scheme, K, N) || scheme == ORC_FP16) return -1;
    const long G = K / ORC_GROUP;
    #pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n) {
        for (long k = 0; k < K; ++k) {
            float s, z;
            if (scheme == ORC_ASYM_GROUP) { s = lpq_oracle_h2f(scales[n * G + k / ORC_GROUP]); z = lpq_oracle_h2f(zeros[n * G + k / ORC_GROUP]); }
            else                          { s = lpq_oracle_h2f(scales[n]); z = 0.0f; }
            volatile float p = s * (float)codes[n * K + k];
            volatile float v = p + z;
            w_deq[n * K + k] = v;
        }
    }
    return 0;
}

/* 16-bit layers: the weights are used as they are. */
int lpq_oracle_fp16_to_f32(const uint16_t *w, long count, float *out)
{
    for (long i = 0; i < count; ++i) out[i] = lpq_oracle_h2f(w[i]);
    return 0;
}

/* ---- O5: y[m][n] = sum_k x[m][k] * w~[n][k] (+ bias[n]) in fp64 ----------------------- */

int lpq_oracle_matmul(const uint16_t *x, const float *w_deq, long M, long K, long N,
                      const uint16_t *bias, double *y)
{
    if (M <= 0 || K <= 0 || N <= 0) return -1;
    #pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n) {
        for (long m = 0; m < M; ++m) {
            double acc = 0.0;
            for (long k = 0; k < K; ++k)
                acc += (double)lpq_oracle_h2f(x[m * K + k]) * (double)w_deq[n * K + k];
            if (bias) acc += (double)lpq_oracle_h2f(bias[n]);
            y[m * N + n] = acc;
        }
    }
    return 0;
}
