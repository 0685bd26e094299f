// The rest of the decoder layer around the four linears: layer normalisation, KV-cache append and
// causal attention over the pre-allocated cache (LLM-PQ, arXiv 2403.01136: Sec. 4.1 "KV Storage
// Modeling" reserves the cache for s + n positions; Sec. 5 serves models with a pre-allocated cache).
// The operators are the published pre-LayerNorm decoder block of the paper's models.
//
// Cache layout per layer: K [B][H][S][d] (a position's d values contiguous) and V transposed,
// VT [B][H][d][S] (a feature's positions contiguous).  With that, both contractions of attention read
// their operands along the contracted index: q.K over d, p.V over positions -- as 16-byte loads, and in
// the prefill kernel directly as MFMA B operands from global memory (no LDS staging, no transposes).
#include <algorithm>
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// block-wide reduction over 256 threads (4 waves); every thread gets the result
template <bool MAX>
__device__ __forceinline__ float block_reduce(float v, float* red /*[4] LDS*/)
{
    v = MAX ? wave_max(v) : wave_sum(v);
    __syncthreads();                                   // red may still be read from a previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return MAX ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : (red[0] + red[1]) + (red[2] + red[3]);
}

// ---- layer normalisation: one workgroup per row, the row held in registers -------------------
// HBM-bound: 2 bytes read + 2 bytes written per element.
constexpr int LN_MAX_CHUNKS = 8;                       // 8 halves per chunk and thread: rows up to 16384

__global__ __launch_bounds__(256) void layernorm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma,
                                                        const uint16_t* __restrict__ beta, float eps, int h, uint16_t* __restrict__ y)
{
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const int nch = h / 8;                             // 16-byte chunks in a row
    float v[LN_MAX_CHUNKS][8];
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < LN_MAX_CHUNKS; ++c) {
        const int ch = threadIdx.x + 256 * c;
        if (ch < nch) {
            const h8 t = *reinterpret_cast<const h8*>(x + row * h + 8 * ch);
#pragma unroll
            for (int e = 0; e < 8; ++e) { v[c][e] = (float)t[e]; s += v[c][e]; }
        }
    }
    const float mean = block_reduce<false>(s, red) / (float)h;
    float q = 0.0f;
#pragma unroll
    for (int c = 0; c < LN_MAX_CHUNKS; ++c)
        if (threadIdx.x + 256 * c < nch)
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = v[c][e] - mean; q += d * d; }
    const float rstd = 1.0f / sqrtf(block_reduce<false>(q, red) / (float)h + eps);
#pragma unroll
    for (int c = 0; c < LN_MAX_CHUNKS; ++c) {
        const int ch = threadIdx.x + 256 * c;
        if (ch < nch) {
            const h8 g = *reinterpret_cast<const h8*>(gamma + 8 * ch), b = *reinterpret_cast<const h8*>(beta + 8 * ch);
            h8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)((v[c][e] - mean) * rstd * (float)g[e] + (float)b[e]);
            *reinterpret_cast<h8*>(y + row * h + 8 * ch) = o;
        }
    }
}

// ---- KV append: the K and V parts of qkv [tokens][3h] into the caches at positions pos0.. -----
// Grid (sequences * heads, ceil(T / 64)): a workgroup moves 64 tokens of one head.  K rows are copied as
// they are; V is transposed through LDS so that a wave writes 64 consecutive positions of one feature row.
template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ kc, uint16_t* __restrict__ vtc,
                                                        int T, int pos0, int H, int S)
{
    __shared__ uint16_t vs[64][D + 2];                 // +2: feature-major reads of a column hit different banks
    typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
    const int bh = blockIdx.x, b = bh / H, head = bh % H, t0 = 64 * blockIdx.y;
    const int h = H * D, nt = min(64, T - t0);
    constexpr int CH = D / 8;                          // 16-byte chunks per token and head
    for (int i = threadIdx.x; i < nt * CH; i += 256) {
        const int t = i / CH, c = i % CH;
        const uint16_t* src = qkv + ((size_t)b * T + t0 + t) * 3 * h + head * D + 8 * c;
        const u16x8 k = *reinterpret_cast<const u16x8*>(src + h), v = *reinterpret_cast<const u16x8*>(src + 2 * h);
        *reinterpret_cast<u16x8*>(kc + (((size_t)b * H + head) * S + pos0 + t0 + t) * D + 8 * c) = k;
#pragma unroll
        for (int e = 0; e < 8; ++e) vs[t][8 * c + e] = v[e];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane < nt)
        for (int dd = wave; dd < D; dd += 4) vtc[(((size_t)b * H + head) * D + dd) * S + pos0 + t0 + lane] = vs[lane][dd];
}

// ---- decode attention: one new token per sequence over L = pos0 + 1 cached positions ------------
// HBM-bound on the cache: 2 * L * d * 2 bytes per (sequence, head).  Grid (sequences * heads, splits);
// a workgroup takes a contiguous range of positions: scores q.K (lanes along d, D/8 lanes per key),
// softmax statistics, then p.V (lanes along positions, one feature row of VT at a time).  With several
// splits the unnormalised partial outputs and their (max, sum) go to a workspace and a second kernel
// combines them.
constexpr int ATT_MAX_RANGE = 2048;                    // positions per workgroup (scores kept in LDS)

template <int D>
__global__ __launch_bounds__(256) void attention_decode_kernel(const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kc,
                                                               const uint16_t* __restrict__ vtc, const float* __restrict__ slopes,
                                                               int H, int S, int L, int range, int splits, uint16_t* __restrict__ out,
                                                               float* __restrict__ part)
{
    __shared__ __attribute__((aligned(16))) float sc[ATT_MAX_RANGE];
    __shared__ float red[4];
    constexpr int LPK = D / 8, KPW = 64 / LPK;         // lanes per key, keys per wave-load
    const int bh = blockIdx.x, b = bh / H, head = bh % H, split = blockIdx.y;
    const int j0 = split * range, j1 = min(L, j0 + range), n = j1 - j0;      // this workgroup's positions [j0, j1)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = H * D;
    const float slope = slopes ? slopes[head] : 0.0f;
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);
    // the lane's 8 query features
    float q[8];
    {
        const h8 t = *reinterpret_cast<const h8*>(qkv + (size_t)b * 3 * h + head * D + 8 * (lane % LPK));
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = (float)t[e];
    }
    const uint16_t* kbase = kc + ((size_t)b * H + head) * S * D;
    // four key rows per lane and round, their loads issued together (positions past the range are clamped
    // to its last one and not stored)
    for (int i0 = wave * KPW + lane / LPK; i0 < n; i0 += 16 * KPW) {
        h8 k[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            k[u] = *reinterpret_cast<const h8*>(kbase + (size_t)(j0 + min(i0 + 4 * KPW * u, n - 1)) * D + 8 * (lane % LPK));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + 4 * KPW * u;
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot += q[e] * (float)k[u][e];
#pragma unroll
            for (int off = LPK / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
            if (lane % LPK == 0 && i < n) sc[i] = dot * inv_sqrt_d + slope * (float)(j0 + i - (L - 1));
        }
    }
    __syncthreads();
    float m = -INFINITY;
    for (int i = tid; i < n; i += 256) m = fmaxf(m, sc[i]);
    m = block_reduce<true>(m, red);
    float l = 0.0f;
    for (int i = tid; i < range; i += 256) {           // weights; zero past the end so that the tail multiplies to zero
        const float p = i < n ? expf(sc[i] - m) : 0.0f;
        sc[i] = p;
        l += p;
    }
    l = block_reduce<false>(l, red);
    __syncthreads();
    // out[dd] = sum_j p[j] * VT[dd][j]; wave w takes rows dd = w, w + 4, ...
    const uint16_t* vbase = vtc + ((size_t)b * H + head) * D * S;
    // four feature rows per wave and round, their loads issued together
    for (int d0 = 4 * wave; d0 < D; d0 += 16) {
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int i = 8 * lane; i < n; i += 512) {
            h8 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const h8*>(vbase + (size_t)(d0 + u) * S + j0 + i);
            const f4 p0 = *reinterpret_cast<const f4*>(&sc[i]), p1 = *reinterpret_cast<const f4*>(&sc[i + 4]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float p = e < 4 ? p0[e] : p1[e - 4];
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[u] += p != 0.0f ? p * (float)v[u][e] : 0.0f;      // positions past L hold anything, also NaN
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float r = wave_sum(acc[u]);
            if (lane == 0) {
                if (splits == 1) out[(size_t)b * h + head * D + d0 + u] = __builtin_bit_cast(uint16_t, (_Float16)(r / l));
                else part[((size_t)bh * splits + split) * (D + 2) + d0 + u] = r;
            }
        }
    }
    if (splits > 1 && tid == 0) {
        float* ps = part + ((size_t)bh * splits + split) * (D + 2);
        ps[D] = m;
        ps[D + 1] = l;
    }
}

template <int D>
__global__ void attention_combine_kernel(const float* __restrict__ part, int splits, uint16_t* __restrict__ out)
{
    const int bh = blockIdx.x, dd = threadIdx.x;       // out is [B][H * D]: row b, column head * D + dd = bh * D + dd
    float m = -INFINITY;
    for (int s = 0; s < splits; ++s) m = fmaxf(m, part[((size_t)bh * splits + s) * (D + 2) + D]);
    float num = 0.0f, den = 0.0f;
    for (int s = 0; s < splits; ++s) {
        const float* ps = part + ((size_t)bh * splits + s) * (D + 2);
        const float w = expf(ps[D] - m);
        num += w * ps[dd];
        den += w * ps[D + 1];
    }
    out[(size_t)bh * D + dd] = __builtin_bit_cast(uint16_t, (_Float16)(num / den));
}

// ---- prefill attention: T new tokens per sequence, causal, over positions 0 .. pos0 + t ----------
// Grid (sequences * heads, ceil(T / 64)); a workgroup takes 64 queries, each wave 16 of them, and
// walks the visible keys 64 at a time with the usual running maximum / sum.  Both products run on
// 16x16x32 MFMAs whose B operands come straight from the caches: S = Q.K^T reads a key's d values,
// O += P.V reads a feature's positions from VT.  Only P changes hands (accumulator layout -> A operand
// layout), through 2 KB of LDS per wave.
template <int D>
__global__ __launch_bounds__(256) void attention_prefill_kernel(const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kc,
                                                                const uint16_t* __restrict__ vtc, const float* __restrict__ slopes,
                                                                int H, int S, int T, int pos0, uint16_t* __restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint16_t pl[4][16][72];      // per wave: P as fp16 [query][key], rows padded to 144 bytes
    constexpr int DC = D / 32;                         // 32-wide chunks of the head dimension
    const int bh = blockIdx.x, b = bh / H, head = bh % H;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 15, kq = lane >> 4;
    const int h = H * D;
    const int t0 = 64 * blockIdx.y + 16 * wave;        // this wave's first query (token index within the sequence)
    const float slope = slopes ? slopes[head] : 0.0f;
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);
    if (t0 >= T) return;                               // whole wave past the end (no workgroup barrier below)
    // A operands of Q: lane (query r, features 32c + 8kq ..)
    h8 qa[DC];
    {
        const int t = min(t0 + r, T - 1);
        const uint16_t* qp = qkv + ((size_t)b * T + t) * 3 * h + head * D + 8 * kq;
#pragma unroll
        for (int c = 0; c < DC; ++c) qa[c] = *reinterpret_cast<const h8*>(qp + 32 * c);
    }
    f4 o[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] = f4{0, 0, 0, 0};
    float m[4], l[4];                                  // running max and sum of the lane's four queries 4kq + v
#pragma unroll
    for (int v = 0; v < 4; ++v) { m[v] = -INFINITY; l[v] = 0.0f; }
    const uint16_t* kbase = kc + ((size_t)b * H + head) * S * D;
    const uint16_t* vbase = vtc + ((size_t)b * H + head) * D * S;
    const int last_pos = pos0 + min(t0 + 15, T - 1);   // the furthest position any query of this wave sees
    const int valid = pos0 + T;                        // cache positions written so far
    for (int j0 = 0; j0 <= last_pos; j0 += 64) {
        // scores of 16 queries x 64 keys: four 16-key tiles
        f4 s[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            s[kt] = f4{0, 0, 0, 0};
            const int key = min(j0 + 16 * kt + r, S - 1);             // B operand: lane (key r, features 32c + 8kq ..)
#pragma unroll
            for (int c = 0; c < DC; ++c) {
                const h8 kb = *reinterpret_cast<const h8*>(kbase + (size_t)key * D + 32 * c + 8 * kq);
                s[kt] = mfma16(qa[c], kb, s[kt]);
            }
        }
        // lane holds scores of queries 4kq + v against keys j0 + 16kt + r
        float mx[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int p = pos0 + t0 + 4 * kq + v;      // the query's position
            mx[v] = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                const int j = j0 + 16 * kt + r;
                const float sv = s[kt][v] * inv_sqrt_d + slope * (float)(j - p);
                s[kt][v] = j <= p ? sv : -INFINITY;    // causal mask (also hides keys past the written positions)
                mx[v] = fmaxf(mx[v], s[kt][v]);
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], off));
        }
        float alpha[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float mn = fmaxf(m[v], mx[v]);       // finite from the first tile on: key 0 is visible to every query
            alpha[v] = expf(m[v] - mn);
            m[v] = mn;
            float rs = 0.0f;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                const float p = expf(s[kt][v] - mn);
                s[kt][v] = p;
                rs += p;
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) rs += __shfl_xor(rs, off);
            l[v] = l[v] * alpha[v] + rs;
        }
#pragma unroll
        for (int i = 0; i < D / 16; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) o[i][v] *= alpha[v];
        // P: accumulator layout -> A operand layout through LDS (wave-private, so no workgroup barrier)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) pl[wave][4 * kq + v][16 * kt + r] = __builtin_bit_cast(uint16_t, (_Float16)s[kt][v]);
        __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): the wave's own LDS writes have landed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < 2; ++c) {                  // two 32-key chunks
            const h8 pa = *reinterpret_cast<const h8*>(&pl[wave][r][32 * c + 8 * kq]);
            const int jb = j0 + 32 * c + 8 * kq;       // the lane's 8 keys of this chunk
#pragma unroll
            for (int i = 0; i < D / 16; ++i) {
                // B operand: lane (feature 16i + r, keys jb ..): 16 bytes of VT
                h8 vb = *reinterpret_cast<const h8*>(vbase + (size_t)(16 * i + r) * S + min(jb, S - 8));
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (jb + e >= valid) vb[e] = (_Float16)0.0f;      // unwritten positions hold anything, also NaN
                o[i] = mfma16(pa, vb, o[i]);
            }
        }
        __builtin_amdgcn_wave_barrier();               // reads of pl done before the next tile overwrites it
    }
    // lane holds queries 4kq + v, features 16i + r
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int t = t0 + 4 * kq + v;
        if (t >= T) continue;
        const float inv = 1.0f / l[v];
        uint16_t* op = out + ((size_t)b * T + t) * h + head * D + r;
#pragma unroll
        for (int i = 0; i < D / 16; ++i) op[16 * i] = __builtin_bit_cast(uint16_t, (_Float16)(o[i][v] * inv));
    }
}

}  // namespace

hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, float eps, int M, int h, void* y, hipStream_t s)
{
    layernorm_kernel<<<(unsigned)M, 256, 0, s>>>(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(gamma),
                                                 static_cast<const uint16_t*>(beta), eps, h, static_cast<uint16_t*>(y));
    return hipGetLastError();
}

int layernorm_max_hidden() { return 256 * 8 * LN_MAX_CHUNKS; }

hipError_t launch_kv_append(const void* qkv, void* kc, void* vtc, int n_seqs, int T, int pos0, int H, int d, int S, hipStream_t s)
{
    const dim3 grid((unsigned)(n_seqs * H), (unsigned)((T + 63) / 64));
    const uint16_t* q = static_cast<const uint16_t*>(qkv);
    if (d == 128) kv_append_kernel<128><<<grid, 256, 0, s>>>(q, static_cast<uint16_t*>(kc), static_cast<uint16_t*>(vtc), T, pos0, H, S);
    else          kv_append_kernel<64><<<grid, 256, 0, s>>>(q, static_cast<uint16_t*>(kc), static_cast<uint16_t*>(vtc), T, pos0, H, S);
    return hipGetLastError();
}

// positions per workgroup and number of splits of a decode-attention launch
void attention_decode_plan(int n_seqs, int H, int L, int* range, int* splits)
{
    const int want = std::max(1, 512 / std::max(1, n_seqs * H));           // enough workgroups for two per CU
    int sp = std::min(want, (L + 63) / 64);
    int rg = ((L + sp - 1) / sp + 63) / 64 * 64;
    if (rg > ATT_MAX_RANGE) rg = ATT_MAX_RANGE;
    sp = (L + rg - 1) / rg;
    *range = rg;
    *splits = sp;
}

size_t attention_decode_workspace_floats(int n_seqs, int H, int d, int splits) { return splits > 1 ? (size_t)n_seqs * H * splits * (d + 2) : 0; }

hipError_t launch_attention(const void* qkv, const void* kc, const void* vtc, const float* slopes, int n_seqs, int T, int pos0, int H, int d,
                            int S, void* out, float* part, hipStream_t s)
{
    const uint16_t* q = static_cast<const uint16_t*>(qkv);
    const uint16_t* k = static_cast<const uint16_t*>(kc);
    const uint16_t* v = static_cast<const uint16_t*>(vtc);
    uint16_t* o = static_cast<uint16_t*>(out);
    if (T == 1) {
        int range, splits;
        attention_decode_plan(n_seqs, H, pos0 + 1, &range, &splits);
        const dim3 grid((unsigned)(n_seqs * H), (unsigned)splits);
        if (d == 128) attention_decode_kernel<128><<<grid, 256, 0, s>>>(q, k, v, slopes, H, S, pos0 + 1, range, splits, o, part);
        else          attention_decode_kernel<64><<<grid, 256, 0, s>>>(q, k, v, slopes, H, S, pos0 + 1, range, splits, o, part);
        if (splits > 1) {
            if (d == 128) attention_combine_kernel<128><<<(unsigned)(n_seqs * H), 128, 0, s>>>(part, splits, o);
            else          attention_combine_kernel<64><<<(unsigned)(n_seqs * H), 64, 0, s>>>(part, splits, o);
        }
    } else {
        const dim3 grid((unsigned)(n_seqs * H), (unsigned)((T + 63) / 64));
        if (d == 128) attention_prefill_kernel<128><<<grid, 256, 0, s>>>(q, k, v, slopes, H, S, T, pos0, o);
        else          attention_prefill_kernel<64><<<grid, 256, 0, s>>>(q, k, v, slopes, H, S, T, pos0, o);
    }
    return hipGetLastError();
}

}  // namespace lpq
