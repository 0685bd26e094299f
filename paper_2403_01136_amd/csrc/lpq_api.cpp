// C-ABI entry points: host-side validation, work decomposition, kernel dispatch.
// Every argument check happens before the first HIP call (see include/lpq.h).
#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "lpq_common.h"

namespace lpq {

int variant_of(const lpq_qdesc& d)
{
    if (d.scheme == LPQ_FP16) return d.bits == 16 ? 4 : -1;
    if (d.scheme == LPQ_ASYM_GROUP) return d.bits == 3 ? 0 : d.bits == 4 ? 1 : d.bits == 8 ? 2 : -1;
    if (d.scheme == LPQ_SYM_CHANNEL) return d.bits == 8 ? 3 : -1;
    return -1;
}

size_t tile_bytes_of(int variant)
{
    static const size_t tb[5] = {768, 1024, 2048, 2048, 4096};
    return tb[variant];
}

namespace {

lpq_status check_desc(const lpq_qdesc* d)
{
    if (!d) return LPQ_ERR_NULL;
    if (d->bits != 3 && d->bits != 4 && d->bits != 8 && d->bits != 16) return LPQ_ERR_BITS;
    if (d->scheme != LPQ_FP16 && d->scheme != LPQ_ASYM_GROUP && d->scheme != LPQ_SYM_CHANNEL) return LPQ_ERR_SCHEME;
    if (variant_of(*d) < 0) return LPQ_ERR_SCHEME;
    if (d->scheme == LPQ_ASYM_GROUP ? d->group_size != 128 : (d->group_size != 0 && d->group_size != 128)) return LPQ_ERR_SCHEME;
    if (d->K <= 0 || d->N <= 0 || d->K % 128 != 0 || d->N % 64 != 0) return LPQ_ERR_SHAPE;
    return LPQ_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

lpq_status check_weight(const lpq_qweight* w)
{
    if (!w) return LPQ_ERR_NULL;
    lpq_status st = check_desc(&w->d);
    if (st != LPQ_OK) return st;
    if (!w->codes) return LPQ_ERR_NULL;
    if (w->d.scheme != LPQ_FP16 && !w->scales) return LPQ_ERR_NULL;
    if (w->d.scheme == LPQ_ASYM_GROUP && !w->zeros) return LPQ_ERR_NULL;
    if (misaligned(w->codes) || (w->d.scheme != LPQ_FP16 && misaligned(w->scales)) ||
        (w->d.scheme == LPQ_ASYM_GROUP && misaligned(w->zeros)) || (w->bias && misaligned(w->bias)))
        return LPQ_ERR_ALIGN;
    return LPQ_OK;
}

// the descriptor a quantiser call is given and the buffers it is to fill
lpq_status check_quantize_target(const lpq_qdesc* desc, const lpq_qweight* out)
{
    lpq_status st = check_desc(desc);
    if (st != LPQ_OK) return st;
    if (out->d.bits != desc->bits || out->d.scheme != desc->scheme || out->d.K != desc->K || out->d.N != desc->N ||
        out->d.group_size != desc->group_size)
        return LPQ_ERR_SHAPE;
    return check_weight(out);
}

lpq_status check_linear(const lpq_qweight* w, const void* x, int32_t M, const void* y)
{
    lpq_status st = check_weight(w);
    if (st != LPQ_OK) return st;
    if (!x || !y) return LPQ_ERR_NULL;
    if (M < 1) return LPQ_ERR_SHAPE;
    if (misaligned(x) || misaligned(y)) return LPQ_ERR_ALIGN;
    return LPQ_OK;
}

// ---- split-K workspace: one block per device, grown on demand.  A block that has been handed out is never
// freed before the process ends: a captured HIP graph, or work still queued on a stream, may hold its address.
// Growth allocates a new block and retires the old one (kept allocated); once lpq_workspace_reserve has been
// called on a device, that device's block no longer grows and a larger need is an error.
struct Workspace {
    std::mutex mu;
    void* ptr[64] = {};
    size_t bytes[64] = {};
    bool reserved[64] = {};
    std::vector<void*> retired;      // earlier blocks, released by the runtime at process exit
};
Workspace g_ws;

// What a request of `need` bytes does to a block of `have` bytes: 0 = reuse it, > 0 = allocate a new block of that
// size; LPQ_ERR_BUFSIZE if a reservation forbids growth.
lpq_status workspace_policy(size_t have, bool reserved, size_t need, size_t* alloc)
{
    *alloc = 0;
    if (need <= have) return LPQ_OK;
    if (reserved) return LPQ_ERR_BUFSIZE;
    *alloc = std::max(need + need / 4, (size_t)8 << 20);
    return LPQ_OK;
}

lpq_status workspace_grow(int dev, size_t want)      // g_ws.mu held
{
    void* fresh = nullptr;
    if (hipMalloc(&fresh, want) != hipSuccess) { (void)hipGetLastError(); return LPQ_ERR_BUFSIZE; }
    if (g_ws.ptr[dev]) g_ws.retired.push_back(g_ws.ptr[dev]);
    g_ws.ptr[dev] = fresh;
    g_ws.bytes[dev] = want;
    return LPQ_OK;
}

lpq_status library_workspace(size_t need, float** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LPQ_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_ws.mu);
    size_t alloc = 0;
    lpq_status st = workspace_policy(g_ws.bytes[dev], g_ws.reserved[dev], need, &alloc);
    if (st != LPQ_OK) return st;
    if (alloc && (st = workspace_grow(dev, alloc)) != LPQ_OK) return st;
    *out = static_cast<float*>(g_ws.ptr[dev]);
    return LPQ_OK;
}

// Partial sums of a call: the library's own workspace, or -- for the entry point that must not allocate -- the
// device's static scratch array (a larger need is an error there, never an allocation).
lpq_status workspace(bool static_ws, size_t need, float** out)
{
    if (!static_ws) return library_workspace(need, out);
    void* p = nullptr;
    size_t bytes = 0;
    if (static_scratch(&p, &bytes) != hipSuccess) { (void)hipGetLastError(); return LPQ_ERR_DEVICE; }
    if (need > bytes) return LPQ_ERR_BUFSIZE;
    *out = static_cast<float*>(p);
    return LPQ_OK;
}

// Compute units of the current device (cached).
lpq_status device_cus(int* out)
{
    static std::mutex mu;
    static int cus[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LPQ_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mu);
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return LPQ_ERR_DEVICE;
        cus[dev] = n;
    }
    *out = cus[dev];
    return LPQ_OK;
}

// Routing of decode launches between the two kernel families (lpq_set_decode_routing; defaults measured on MI355X).
std::atomic<int32_t> g_rows_max_mb{192};     // launches that stream at most this many MiB of codes take the small-launch kernel
std::atomic<int32_t> g_rows_tiles{0};        // 2..5: force that many 16-row tiles per workgroup there; 0: the planner's choice

// Wavefronts per decode workgroup: eight, one workgroup per CU (two waves per SIMD), so that a step's activations
// are staged once for 512 rows of W.  (Four waves and two workgroups per CU move twice the activation bytes from
// L2 -- a third of the weight bytes at 3 bits and 16 token rows -- and measured 0.5-4 % slower on every configuration.)
// The workgroups per launch are what the chip holds at once.
int decode_waves(int /*M*/) { return 8; }

lpq_status decode_block_count(int waves, int* out)
{
    int cus = 0;
    lpq_status st = device_cus(&cus);
    if (st != LPQ_OK) return st;
    *out = cus * (8 / waves);
    return LPQ_OK;
}

// relative cost of streaming one byte of each variant (x16), used to weight the even-share split
uint32_t variant_cost_x16(int variant)
{
    // measured on MI355X: bytes of 3- and 4-bit codes take longer to stream because unpacking them is
    // ALU work per byte; 8-bit codes and fp16 weights run at the memory system's pace
    static const uint32_t c[5] = {26, 21, 17, 17, 16};
    return c[variant];
}

// Workgroup shape of a single linear in the small-launch decode kernel: 16-row tiles per workgroup (T) and K
// splits (s).  Measured on MI355X (OPT-13B, 7B- and 70B-class shapes, 3- and 4-bit): a launch runs fastest
// when its workgroups just fit the compute units once -- a unit that gets two takes 2.6 times as long, not
// twice -- and a workgroup's time grows with its steps times (the activations it reads per step, from L2,
// plus T tiles of weights).  T = 3 and 5 cut a 64-row block across workgroups (e.g. 1280 tiles = 256 x 5);
// at T = 5 the kernel holds the whole register file and runs a third slower per byte.  A split costs a second
// kernel.  The estimate below (microseconds) is only used to rank the choices.
void rows_plan(const LinDesc& L, int tok_tiles, int cus, int* tiles, int* splits)
{
    static const double tile_us[5] = {0.024, 0.032, 0.064, 0.064, 0.128};     // per tile and step, by variant
    const int KT = L.kt, n_tiles = L.N / 16;
    double best = 1e30;
    *tiles = 4;
    *splits = 1;
    static const int order[4] = {4, 2, 3, 5};                                // ties go to the earlier entry
    for (int oi = 0; oi < 4; ++oi) {
        const int T = order[oi];
        if (L.variant == 4 && T > 2 && T != 4) continue;                     // fp16 weights: one or two tiles (4 stands for 2)
        const int rt = (L.variant == 4 && T > 2) ? 2 : T;
        if (n_tiles % rt != 0) continue;
        const double step_us = 0.06 * tok_tiles + rt * tile_us[L.variant] + (rt == 5 ? 0.09 : 0.0);
        for (int s = 1; s <= 8; ++s) {
            const long wgs = (long)(n_tiles / rt) * s;
            // a split is there to fill the chip, not to add rounds; a wave wants several steps per stage of its ring
            if (s > 1 && (KT / s < 16 || wgs > cus)) break;
            const long rounds = (wgs + cus - 1) / cus;
            const double est = (rounds == 1 ? 1.0 : 1.3 * rounds) * ((KT + s - 1) / s) * step_us + (s > 1 ? 5.0 : 0.0);
            if (est < best * 0.98) best = est, *tiles = T, *splits = s;
        }
    }
}

// Bytes that decode_prepare_kernel leaves for a linear in a decode launch of up to 32 token rows per pass.  The group
// sums: per token row (32 of them) an fp16 pair per 128-column group, groups padded to a multiple of 16, and 16 bytes
// for the row's factors; behind them, for 3-bit weights that the launch reads in place, `rows` rows of scaled
// activations.
size_t prepared_bytes(const lpq_qdesc& d, int rows, bool in_place)
{
    const size_t sums = (size_t)32 * (4 * (((size_t)d.K / 128 + 15) & ~(size_t)15) + 16);
    return sums + (in_place && variant_of(d) == 0 ? (size_t)rows * (size_t)d.K * 2 : 0);
}

struct LinearCall {
    const lpq_qweight* w;
    const void* x;
    void* y;
    const void* residual = nullptr;
    int32_t act = LPQ_ACT_NONE;
};

// Whether a stage-wide decode launch of M token rows reads its 3-bit codes in place (lpq_decode.hip: a third of the
// unpacking instructions less, against a copy of those linears' activations scaled beforehand).  The copy costs by
// the row, the saving is per weight: it pays at up to 16 rows where 3-bit weights are a good part of what the launch
// streams.  Measured: +2.5 % (16 rows) to +5 % (1 row) on an all-3-bit stage, +0.5 % on one of alternating 3- and
// 4-bit layers, -0.6 % where an eighth of the bytes is 3-bit; at 32 rows -3 to -5 %.
bool reads_in_place(const std::vector<LinearCall>& calls, size_t begin, size_t end, int32_t M)
{
    if (M > 16) return false;
    double w3 = 0.0, all = 0.0;
    for (size_t c = begin; c < end; ++c) {
        const lpq_qdesc& d = calls[c].w->d;
        const double bytes = (double)d.K * (double)d.N * d.bits;
        all += bytes;
        if (variant_of(d) == 0) w3 += bytes;
    }
    return w3 >= 0.25 * all;
}

// Decode-phase dispatch of a list of independent linears: grouped launches of at most
// MAX_LIN_PER_LAUNCH linears, 64 token rows per pass, each launch one round of equally loaded
// workgroups (see lpq_decode.hip).
lpq_status run_decode(const std::vector<LinearCall>& calls, int32_t M, hipStream_t stream, bool static_ws = false)
{
    const size_t n = calls.size();
    const size_t n_launch = (n + MAX_LIN_PER_LAUNCH - 1) / MAX_LIN_PER_LAUNCH;
    const size_t per_launch = (n + n_launch - 1) / n_launch;
    const int waves = decode_waves(M);
    int n_blocks = 0;
    lpq_status st = decode_block_count(waves, &n_blocks);
    if (st != LPQ_OK) return st;
    const int tok_rows = std::min(64, (M + 15) / 16 * 16);
    const int slot_floats = tok_rows * waves * 64;
    // after the partial tiles: what decode_prepare_kernel leaves for one launch whose last pass has up to 32 token
    // rows; launches and passes run one after the other on the stream and share the space
    const size_t partial_bytes = ((size_t)2 * n_blocks * slot_floats * sizeof(float) + 255) & ~(size_t)255;
    const int last_rows = (M - 1) % 64 + 1;
    size_t sums_bytes = 0;
    if (last_rows <= 32)
        for (size_t li = 0; li < n_launch; ++li) {
            size_t b = 0;
            const size_t c0 = li * per_launch, c1 = std::min(n, (li + 1) * per_launch);
            const bool in_place = reads_in_place(calls, c0, c1, M);
            for (size_t c = c0; c < c1; ++c) b += prepared_bytes(calls[c].w->d, last_rows, in_place);
            sums_bytes = std::max(sums_bytes, b);
        }
    float* ws = nullptr;
    st = workspace(static_ws, partial_bytes + sums_bytes, &ws);
    if (st != LPQ_OK) return st;
    for (size_t li = 0; li < n_launch; ++li) {
        DecodeArgs a;
        a.M = M;
        a.m0 = 0;
        a.n_lin = 0;
        a.waves = waves;
        a.n_blocks = n_blocks;
        a.slot_floats = slot_floats;
        a.row_tiles = 4;
        a.pad = 0;
        a.partial = ws;
        a.prep = sums_bytes ? reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(ws) + partial_bytes) : nullptr;
        uint64_t total = 0;
        size_t sums_off16 = 0;               // in 16-byte units
        const bool in_place = reads_in_place(calls, li * per_launch, std::min(n, (li + 1) * per_launch), M);
        for (size_t c = li * per_launch; c < std::min(n, (li + 1) * per_launch); ++c) {
            const lpq_qweight& w = *calls[c].w;
            LinDesc& L = a.lin[a.n_lin++];
            L.codes = static_cast<const uint8_t*>(w.codes);
            L.scales = static_cast<const uint16_t*>(w.scales);
            L.zeros = static_cast<const uint16_t*>(w.zeros);
            L.x = static_cast<const uint16_t*>(calls[c].x);
            L.y = static_cast<uint16_t*>(calls[c].y);
            L.bias = static_cast<const uint16_t*>(w.bias);
            L.residual = static_cast<const uint16_t*>(calls[c].residual);
            L.act = (uint8_t)calls[c].act;
            L.aux = (int32_t)sums_off16;
            sums_off16 += prepared_bytes(w.d, last_rows, in_place) / 16;
            if (w.d.K / 128 > 0xffff) return LPQ_ERR_UNSUPPORTED;          // the descriptor keeps K / 128 in 16 bits
            L.kt = (uint16_t)(w.d.K / 128);
            L.N = w.d.N;
            L.variant = (uint8_t)variant_of(w.d);
            const int rows = decode_rows_per_wave(L.variant);
            const uint32_t step_bytes = (uint32_t)(waves * rows) * (128u * (uint32_t)w.d.bits / 8u + (w.d.scheme == LPQ_ASYM_GROUP ? 4u : 0u));
            L.step_weight = step_bytes * variant_cost_x16(L.variant);
            L.cum_weight = total;
            total += (uint64_t)L.step_weight * (uint64_t)lin_row_superblocks(L, waves) * (uint64_t)L.kt;
        }
        if (total >= ((uint64_t)1 << 50)) return LPQ_ERR_UNSUPPORTED;
        a.total_weight = total;
        // A launch that streams little (a single linear of a decoder layer) has too few steps to spread evenly:
        // it goes to the kernel that gives every group of 16-row tiles a workgroup whose waves split K (no fix-up
        // pass), up to 32 token rows per pass.
        const int64_t rows_max_bytes = (int64_t)g_rows_max_mb.load() << 20;
        int64_t stream_bytes = 0;
        for (size_t c = li * per_launch; c < std::min(n, (li + 1) * per_launch); ++c)
            stream_bytes += (int64_t)calls[c].w->d.K * calls[c].w->d.N * calls[c].w->d.bits / 8;
        // 33-64 token rows take two passes of that kernel if the weights are few enough (128 MB) for the second
        // pass to find most of them in the caches; measured on a decoder layer, 7-15 % faster than the even-share kernel.
        if (stream_bytes <= rows_max_bytes && (M <= 32 || (M <= 64 && stream_bytes <= std::min<int64_t>(rows_max_bytes, (int64_t)128 << 20)))) {
            // longest K first: the last workgroups to start are then the shortest
            std::stable_sort(a.lin, a.lin + a.n_lin, [](const LinDesc& x, const LinDesc& y) { return x.kt > y.kt; });
            int cus = 0;
            st = device_cus(&cus);
            if (st != LPQ_OK) return st;
            // 32 token rows per pass (33-64 rows: two passes, the second reads the weights again, mostly from the caches)
            for (int m0 = 0; m0 < M; m0 += 32) {
                DecodeArgs p = a;
                p.M = std::min(32, M - m0);
                p.m0 = 0;
                for (int i = 0; i < p.n_lin; ++i) {
                    LinDesc& L = p.lin[i];
                    L.x += (size_t)m0 * L.K();
                    L.y += (size_t)m0 * L.N;
                    if (L.residual) L.residual += (size_t)m0 * L.N;
                }
                const int tok_tiles = p.M <= 16 ? 1 : 2;
                int tiles = 4, splits1 = 0;
                if (p.n_lin == 1) rows_plan(p.lin[0], tok_tiles, cus, &tiles, &splits1);
                const int forced = g_rows_tiles.load();
                if (forced >= 2 && forced <= 5 && forced != tiles) tiles = forced, splits1 = 0;
                auto group_tiles = [&](const LinDesc& L) { return rows_group_tiles(L.variant, tiles); };
                for (int i = 0; i < p.n_lin; ++i)
                    if ((p.lin[i].N / 16) % group_tiles(p.lin[i]) != 0) tiles = 4, splits1 = 0;    // groups must tile every linear exactly
                int64_t blocks = 0, row_blocks = 0;
                for (int i = 0; i < p.n_lin; ++i) row_blocks += p.lin[i].N / 16 / group_tiles(p.lin[i]);
                int64_t partial_floats = 0;
                for (int i = 0; i < p.n_lin; ++i) {
                    LinDesc& L = p.lin[i];
                    // K splits (L.aux) of a launch of several linears: only if it leaves most compute units without a
                    // workgroup, and only down to 32 steps per workgroup
                    const int KT = L.kt;
                    const int want = (int)std::max<int64_t>(1, 320 / std::max<int64_t>(1, row_blocks));
                    L.aux = splits1 > 0 ? splits1 : std::max(1, std::min(std::min(want, KT / 32), 8));
                    L.step_weight = (uint32_t)partial_floats;             // float offset of this linear's partial sums
                    if (L.aux > 1) partial_floats += (int64_t)L.aux * 16 * tok_tiles * L.N;
                    L.cum_weight = (uint64_t)blocks;
                    blocks += (int64_t)rows_row_blocks(L, tiles) * L.aux;
                }
                if (blocks > 0x7fffffffLL || partial_floats > 0x7fffffffLL) return LPQ_ERR_UNSUPPORTED;
                if (partial_floats) {
                    st = workspace(static_ws, (size_t)partial_floats * sizeof(float), &ws);
                    if (st != LPQ_OK) return st;
                }
                p.partial = ws;
                p.n_blocks = (int32_t)blocks;
                p.row_tiles = tiles;
                p.waves = (blocks <= 64 && tok_tiles == 1) ? 8 : 4;      // very few blocks: more waves per block keep more loads in flight
                if (launch_decode_rows(p, stream) != hipSuccess) return LPQ_ERR_DEVICE;
            }
            continue;
        }
        // A small launch (one linear of a decoder layer) is not cut into more ranges than it has chunks of
        // steps: thinner ranges stream no faster and only multiply the pieces the fix-up pass has to add.
        const int min_steps = M <= 16 ? 16 : 8;              // a 64-token step is 3x as long
        int64_t steps = 0;
        for (int i = 0; i < a.n_lin; ++i) steps += (int64_t)lin_row_superblocks(a.lin[i], waves) * a.lin[i].kt;
        a.n_blocks = (int32_t)std::max<int64_t>(1, std::min<int64_t>(n_blocks, steps / min_steps));
        a.range_q = a.total_weight / (uint64_t)a.n_blocks;
        a.range_rem = (uint32_t)(a.total_weight % (uint64_t)a.n_blocks);
        if (in_place)
            for (int i = 0; i < a.n_lin; ++i)
                if (a.lin[i].variant == 0) a.lin[i].variant = V_W3_INPLACE;
        for (int m0 = 0; m0 < M; m0 += 64) {
            a.m0 = m0;
            if (launch_decode(a, stream) != hipSuccess) return LPQ_ERR_DEVICE;
        }
    }
    return LPQ_OK;
}

// How many groups to split a linear's token blocks into (see PrefillLin).  With g groups, a linear's
// weights are fetched into g of the 8 L2s and its activations into 8 / g of them.  Measured on whole
// stages (OPT-13B and 70B-class shapes, every variant), two groups are best or within 1% of it;
// other counts are for shapes with too few token or row blocks, or that two groups would spread
// unevenly over the XCDs.
int prefill_token_groups(int m_blocks, int n_blocks)
{
    static const int order[4] = {2, 4, 1, 8};
    int best = 1;
    double best_imbalance = 1e30;
    for (int i = 0; i < 4; ++i) {
        const int g = order[i];
        if (g > 1 && (g > m_blocks || 8 / g > n_blocks)) continue;
        const double imbalance = 8.0 * prefill_xcd_tiles(m_blocks, n_blocks, g) / ((double)m_blocks * n_blocks);
        if (imbalance <= 1.15) return g;
        if (imbalance < best_imbalance) { best = g; best_imbalance = imbalance; }
    }
    return best;
}

// K splits of one prefill linear that is launched with too few tiles to fill the chip (a single linear of a
// decoder layer at a small micro-batch; a K = 4h linear whose tiles are four times as long as its launch's
// others).  Estimated time of s splits, in units of one 128-column step of a tile: rounds of workgroups over
// the compute units times steps per workgroup, plus writing and re-reading s fp32 copies of the output
// (8 bytes per element and split; measured ~10 TB/s, most of it served by the caches, against ~4.1 us per
// step) and the second kernel's launch.  Fitted to sweeps of the split count over OPT-13B's four shapes at
// 256-4096 tokens: the choice is the best measured one or within a few per cent of it.
int prefill_k_splits(int tiles, int KT, int32_t M, int32_t N, int cus)
{
    if (tiles >= 2 * cus) return 1;
    static const int cand[7] = {1, 2, 3, 4, 5, 6, 8};
    int best = 1;
    double best_cost = 1e30;
    for (int i = 0; i < 7; ++i) {
        const int s = cand[i];
        if (s > 1 && KT / s < 8) break;                                    // keep the pipeline's fill and drain small
        const double rounds = (double)(((long)tiles * s + cus - 1) / cus);
        double cost = rounds * (double)((KT + s - 1) / s);
        if (s > 1) cost += 8.0 * s * (double)M * (double)N / 1.0e13 / 4.1e-6 + 1.0;
        if (cost < best_cost * 0.97) best_cost = cost, best = s;          // a split must pay clearly
    }
    return best;
}

// Prefill-phase dispatch of a list of independent linears: one grouped launch per storage variant
// (and per MAX_PREFILL_LIN linears), tiles of the longest-K linears first.
lpq_status run_prefill_rows(const std::vector<LinearCall>& calls, int32_t M, int BM, hipStream_t stream, bool static_ws)
{
    int cus = 0;
    lpq_status cst = device_cus(&cus);
    if (cst != LPQ_OK) return cst;
    for (int variant = 0; variant < 5; ++variant) {
        const int m_blocks = (M + BM - 1) / BM;
        std::vector<const LinearCall*> mine;
        for (const LinearCall& c : calls)
            if (variant_of(c.w->d) == variant) mine.push_back(&c);
        std::stable_sort(mine.begin(), mine.end(), [](const LinearCall* a, const LinearCall* b) { return a->w->d.K > b->w->d.K; });
        for (size_t first = 0; first < mine.size(); first += MAX_PREFILL_LIN) {
            PrefillArgs a;
            a.M = M;
            a.n_lin = 0;
            a.tokens_per_tile = BM;
            long tiles = 0, launch_tiles = 0;
            size_t partial_floats = 0;
            for (size_t i = first; i < std::min(mine.size(), first + (size_t)MAX_PREFILL_LIN); ++i)
                launch_tiles += (long)m_blocks * ((mine[i]->w->d.N + 255) / 256);
            for (size_t i = first; i < std::min(mine.size(), first + (size_t)MAX_PREFILL_LIN); ++i) {
                const lpq_qweight& w = *mine[i]->w;
                PrefillLin& L = a.lin[a.n_lin++];
                L.codes = static_cast<const uint8_t*>(w.codes);
                L.scales = static_cast<const uint16_t*>(w.scales);
                L.zeros = static_cast<const uint16_t*>(w.zeros);
                L.x = static_cast<const uint16_t*>(mine[i]->x);
                L.y = static_cast<uint16_t*>(mine[i]->y);
                L.bias = static_cast<const uint16_t*>(w.bias);
                L.residual = static_cast<const uint16_t*>(mine[i]->residual);
                L.act = mine[i]->act;
                L.K = w.d.K;
                L.N = w.d.N;
                L.n_blocks = (w.d.N + 255) / 256;
                L.token_groups = prefill_token_groups(m_blocks, L.n_blocks);
                L.tile_begin = (int32_t)tiles;
                L.pad = 0;
                // splitting is judged per launch: a launch with many tiles fills the chip whatever its linears' shapes
                L.k_splits = launch_tiles >= 2L * cus ? 1 : prefill_k_splits((int)launch_tiles, w.d.K / 128, M, w.d.N, cus);
                L.partial = nullptr;
                if (L.k_splits > 1) partial_floats += (size_t)L.k_splits * M * w.d.N;
                tiles += 8L * L.k_splits * prefill_xcd_tiles(m_blocks, L.n_blocks, L.token_groups);
            }
            if (tiles > 0x7fffffffL) return LPQ_ERR_UNSUPPORTED;
            a.total_tiles = (int32_t)tiles;
            if (partial_floats) {
                float* ws = nullptr;
                lpq_status st = workspace(static_ws, partial_floats * sizeof(float), &ws);
                if (st != LPQ_OK) return st;
                for (int i = 0; i < a.n_lin; ++i) {
                    if (a.lin[i].k_splits <= 1) continue;
                    a.lin[i].partial = ws;
                    ws += (size_t)a.lin[i].k_splits * M * a.lin[i].N;
                }
            }
            if (launch_prefill(variant, a, stream) != hipSuccess) return LPQ_ERR_DEVICE;
        }
    }
    return LPQ_OK;
}

// Tokens per tile.  256 as a rule: weights are fetched and unpacked once per token block.  A call of at most 128 rows
// has one block either way and takes 128-token tiles (half the matrix instructions per step).  A call of 1024 rows
// or more whose last block of 256 would hold at most 128 rows pays a full tile of matrix instructions for that block
// (1100 rows cost what 1280 do): there the tail runs as launches of its own with 128-token tiles -- measured on an
// OPT-13B layer's four linears, 11-19 % less time at 1100, 1152, 1600, 2100 and 3200 rows.  Below 1024 rows a call
// is short of tiles either way, and both a tail launch and 128-token tiles throughout measured slower than the
// ragged block (384 rows: 0.45 against 0.41 ms), so it keeps 256-token tiles.
lpq_status run_prefill(const std::vector<LinearCall>& calls, int32_t M, hipStream_t stream, bool static_ws = false)
{
    const int32_t tail = M % 256, body = M - tail;
    if (M <= 128) return run_prefill_rows(calls, M, 128, stream, static_ws);
    if (tail == 0 || tail > 128) return run_prefill_rows(calls, M, 256, stream, static_ws);
    if (M < 1024) return run_prefill_rows(calls, M, 256, stream, static_ws);
    lpq_status st = run_prefill_rows(calls, body, 256, stream, static_ws);
    if (st != LPQ_OK) return st;
    std::vector<LinearCall> rest(calls);
    for (LinearCall& c : rest) {
        c.x = static_cast<const uint16_t*>(c.x) + (size_t)body * c.w->d.K;
        c.y = static_cast<uint16_t*>(c.y) + (size_t)body * c.w->d.N;
        if (c.residual) c.residual = static_cast<const uint16_t*>(c.residual) + (size_t)body * c.w->d.N;
    }
    return run_prefill_rows(rest, tail, 128, stream, static_ws);
}

lpq_status check_attention_args(const lpq_layer_cfg* cfg, const lpq_layer_state* st, int32_t n_seqs, int32_t T, int32_t pos0)
{
    if (!st->k_cache || !st->vt_cache) return LPQ_ERR_NULL;
    if (cfg->n_heads < 1 || (cfg->head_dim != 64 && cfg->head_dim != 128) || cfg->max_seq < 64 || cfg->max_seq % 64 != 0) return LPQ_ERR_SHAPE;
    if (n_seqs < 1 || T < 1 || pos0 < 0 || (int64_t)pos0 + T > cfg->max_seq) return LPQ_ERR_SHAPE;
    if (misaligned(st->k_cache) || misaligned(st->vt_cache) || (reinterpret_cast<uintptr_t>(st->alibi_slopes) & 3u)) return LPQ_ERR_ALIGN;
    return LPQ_OK;
}

lpq_status run_attention(const void* qkv, const lpq_layer_cfg* cfg, const lpq_layer_state* st, int32_t n_seqs, int32_t T, int32_t pos0,
                         void* out, hipStream_t stream)
{
    float* part = nullptr;
    if (T == 1) {
        int range = 0, splits = 0;
        attention_decode_plan(n_seqs, cfg->n_heads, pos0 + 1, &range, &splits);
        const size_t floats = attention_decode_workspace_floats(n_seqs, cfg->n_heads, cfg->head_dim, splits);
        if (floats) {
            lpq_status s = workspace(false, floats * sizeof(float), &part);
            if (s != LPQ_OK) return s;
        }
    }
    return launch_attention(qkv, st->k_cache, st->vt_cache, st->alibi_slopes, n_seqs, T, pos0, cfg->n_heads, cfg->head_dim, cfg->max_seq,
                            out, part, stream) == hipSuccess ? LPQ_OK : LPQ_ERR_DEVICE;
}

}  // namespace
}  // namespace lpq

using namespace lpq;

extern "C" {

lpq_status lpq_packed_sizes(const lpq_qdesc* desc, size_t* code_bytes, size_t* scale_bytes, size_t* zero_bytes)
{
    if (!desc || !code_bytes || !scale_bytes || !zero_bytes) return LPQ_ERR_NULL;
    lpq_status st = check_desc(desc);
    if (st != LPQ_OK) return st;
    const size_t K = (size_t)desc->K, N = (size_t)desc->N;
    *code_bytes = K * N * (size_t)desc->bits / 8;
    *scale_bytes = desc->scheme == LPQ_ASYM_GROUP ? N * (K / 128) * 2 : desc->scheme == LPQ_SYM_CHANNEL ? N * 2 : 0;
    *zero_bytes = desc->scheme == LPQ_ASYM_GROUP ? *scale_bytes : 0;
    return LPQ_OK;
}

lpq_status lpq_quantize_pack(const void* w_fp16, const lpq_qdesc* desc, lpq_qweight* out, void* hip_stream)
{
    if (!w_fp16 || !desc || !out) return LPQ_ERR_NULL;
    lpq_status st = check_quantize_target(desc, out);
    if (st != LPQ_OK) return st;
    if (misaligned(w_fp16)) return LPQ_ERR_ALIGN;
    return launch_quantize_pack(w_fp16, *desc, 0, desc->N, *out, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? LPQ_OK : LPQ_ERR_DEVICE;
}

lpq_status lpq_quantize_pack_rows(const void* w_rows_fp16, const lpq_qdesc* desc, int32_t row0, int32_t n_rows, lpq_qweight* out,
                                  void* hip_stream)
{
    if (!w_rows_fp16 || !desc || !out) return LPQ_ERR_NULL;
    lpq_status st = check_quantize_target(desc, out);
    if (st != LPQ_OK) return st;
    if (row0 < 0 || n_rows < 0 || row0 % 64 != 0 || n_rows % 64 != 0 || (int64_t)row0 + n_rows > desc->N) return LPQ_ERR_SHAPE;
    if (misaligned(w_rows_fp16)) return LPQ_ERR_ALIGN;
    return launch_quantize_pack(w_rows_fp16, *desc, row0, n_rows, *out, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? LPQ_OK : LPQ_ERR_DEVICE;
}

lpq_status lpq_load_quantize_pack(const void* w_fp16_host, const lpq_qdesc* desc, lpq_qweight* out, void* staging, size_t staging_bytes,
                                  void* hip_stream)
{
    if (!w_fp16_host || !desc || !out || !staging) return LPQ_ERR_NULL;
    lpq_status st = check_quantize_target(desc, out);
    if (st != LPQ_OK) return st;
    if (misaligned(w_fp16_host) || misaligned(staging)) return LPQ_ERR_ALIGN;
    // Bands of rows alternate on the caller's stream: copy a band into the staging buffer, quantise it into
    // its place, copy the next.  The quantiser runs some thirty times faster than the host link, so the copy
    // engine idles 2-3 % of the time; a second stream that overlapped the two was measured at +1 % at best and
    // at -35 % in a runtime state seen after large allocations had been freed, so it is not used.
    const size_t row_bytes = (size_t)desc->K * 2;
    const int64_t chunk_rows = std::min<int64_t>((int64_t)(staging_bytes / row_bytes) / 64 * 64, desc->N);
    if (chunk_rows < 64) return LPQ_ERR_BUFSIZE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (int64_t row = 0; row < desc->N; row += chunk_rows) {
        const int64_t rows = std::min<int64_t>(chunk_rows, desc->N - row);
        if (hipMemcpyAsync(staging, static_cast<const uint8_t*>(w_fp16_host) + (size_t)row * row_bytes, (size_t)rows * row_bytes,
                           hipMemcpyHostToDevice, stream) != hipSuccess)
            return LPQ_ERR_DEVICE;
        if (launch_quantize_pack(staging, *desc, row, rows, *out, stream) != hipSuccess) return LPQ_ERR_DEVICE;
    }
    return LPQ_OK;
}

lpq_status lpq_layernorm(const void* x, const void* gamma, const void* beta, float eps, int32_t M, int32_t hidden, void* y, void* hip_stream)
{
    if (!x || !gamma || !beta || !y) return LPQ_ERR_NULL;
    if (M < 1 || hidden < 8 || hidden % 8 != 0 || hidden > layernorm_max_hidden() || !(eps >= 0.0f)) return LPQ_ERR_SHAPE;
    if (misaligned(x) || misaligned(gamma) || misaligned(beta) || misaligned(y)) return LPQ_ERR_ALIGN;
    return launch_layernorm(x, gamma, beta, eps, M, hidden, y, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? LPQ_OK : LPQ_ERR_DEVICE;
}

lpq_status lpq_kv_append(const void* qkv, const lpq_layer_cfg* cfg, const lpq_layer_state* st, int32_t n_seqs, int32_t T, int32_t pos0,
                         void* hip_stream)
{
    if (!qkv || !cfg || !st) return LPQ_ERR_NULL;
    lpq_status s = check_attention_args(cfg, st, n_seqs, T, pos0);
    if (s != LPQ_OK) return s;
    if (misaligned(qkv)) return LPQ_ERR_ALIGN;
    return launch_kv_append(qkv, st->k_cache, st->vt_cache, n_seqs, T, pos0, cfg->n_heads, cfg->head_dim, cfg->max_seq,
                            static_cast<hipStream_t>(hip_stream)) == hipSuccess ? LPQ_OK : LPQ_ERR_DEVICE;
}

lpq_status lpq_attention(const void* qkv, const lpq_layer_cfg* cfg, const lpq_layer_state* st, int32_t n_seqs, int32_t T, int32_t pos0,
                         void* out, void* hip_stream)
{
    if (!qkv || !cfg || !st || !out) return LPQ_ERR_NULL;
    lpq_status s = check_attention_args(cfg, st, n_seqs, T, pos0);
    if (s != LPQ_OK) return s;
    if (misaligned(qkv) || misaligned(out)) return LPQ_ERR_ALIGN;
    return run_attention(qkv, cfg, st, n_seqs, T, pos0, out, static_cast<hipStream_t>(hip_stream));
}

size_t lpq_decoder_layer_workspace(const lpq_layer* layer, const lpq_layer_cfg* cfg, int32_t M)
{
    if (!layer || !cfg || M < 1 || cfg->n_heads < 1 || cfg->head_dim < 1) return 0;
    const size_t h = (size_t)cfg->n_heads * cfg->head_dim, f = (size_t)std::max(layer->fc1.d.N, 0);
    return (size_t)M * (5 * h + f) * 2;       // h1 / h2, qkv (3h), attention output, feed-forward activations
}

lpq_status lpq_decoder_layer(const lpq_layer* layer, const lpq_layer_cfg* cfg, const lpq_layer_state* st, lpq_phase phase, int32_t n_seqs,
                             int32_t T, int32_t pos0, const void* x, void* y, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!layer || !cfg || !st || !x || !y || !workspace) return LPQ_ERR_NULL;
    if (phase != LPQ_PREFILL && phase != LPQ_DECODE) return LPQ_ERR_UNSUPPORTED;
    if (cfg->activation != LPQ_ACT_NONE && cfg->activation != LPQ_ACT_RELU && cfg->activation != LPQ_ACT_GELU_TANH) return LPQ_ERR_UNSUPPORTED;
    lpq_status s = check_attention_args(cfg, st, n_seqs, T, pos0);
    if (s != LPQ_OK) return s;
    if (!st->ln1_gamma || !st->ln1_beta || !st->ln2_gamma || !st->ln2_beta) return LPQ_ERR_NULL;
    const lpq_qweight* w[4] = {&layer->qkv, &layer->out, &layer->fc1, &layer->fc2};
    for (int j = 0; j < 4; ++j) {
        s = check_weight(w[j]);
        if (s != LPQ_OK) return s;
    }
    const int64_t h = (int64_t)cfg->n_heads * cfg->head_dim, f = layer->fc1.d.N, M = (int64_t)n_seqs * T;
    if (h > layernorm_max_hidden() || M > 0x7fffffff) return LPQ_ERR_SHAPE;
    if (layer->qkv.d.K != h || layer->qkv.d.N != 3 * h || layer->out.d.K != h || layer->out.d.N != h || layer->fc1.d.K != h ||
        layer->fc2.d.K != f || layer->fc2.d.N != h)
        return LPQ_ERR_SHAPE;
    if (misaligned(x) || misaligned(y) || misaligned(workspace) || misaligned(st->ln1_gamma) || misaligned(st->ln1_beta) ||
        misaligned(st->ln2_gamma) || misaligned(st->ln2_beta))
        return LPQ_ERR_ALIGN;
    if (workspace_bytes < lpq_decoder_layer_workspace(layer, cfg, (int32_t)M)) return LPQ_ERR_BUFSIZE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint16_t* h1 = static_cast<uint16_t*>(workspace);          // LN1 output, later LN2 output
    uint16_t* qkv = h1 + M * h;
    uint16_t* att = qkv + 3 * M * h;
    uint16_t* ff = att + M * h;
    auto linear = [&](const lpq_qweight* wt, const void* in, void* out, const void* residual, int act) {
        std::vector<LinearCall> calls(1, LinearCall{wt, in, out, residual, act});
        return phase == LPQ_PREFILL ? run_prefill(calls, (int32_t)M, stream) : run_decode(calls, (int32_t)M, stream);
    };
    if (launch_layernorm(x, st->ln1_gamma, st->ln1_beta, cfg->ln_eps, (int)M, (int)h, h1, stream) != hipSuccess) return LPQ_ERR_DEVICE;
    if ((s = linear(&layer->qkv, h1, qkv, nullptr, LPQ_ACT_NONE)) != LPQ_OK) return s;
    if (launch_kv_append(qkv, st->k_cache, st->vt_cache, n_seqs, T, pos0, cfg->n_heads, cfg->head_dim, cfg->max_seq, stream) != hipSuccess)
        return LPQ_ERR_DEVICE;
    if ((s = run_attention(qkv, cfg, st, n_seqs, T, pos0, att, stream)) != LPQ_OK) return s;
    if ((s = linear(&layer->out, att, y, x, LPQ_ACT_NONE)) != LPQ_OK) return s;                    // y = x + out-projection
    if (launch_layernorm(y, st->ln2_gamma, st->ln2_beta, cfg->ln_eps, (int)M, (int)h, h1, stream) != hipSuccess) return LPQ_ERR_DEVICE;
    if ((s = linear(&layer->fc1, h1, ff, nullptr, cfg->activation)) != LPQ_OK) return s;
    return linear(&layer->fc2, ff, y, y, LPQ_ACT_NONE);                                           // y += feed-forward
}

lpq_status lpq_variance_indicator(const void* w_fp16, int32_t K, int32_t N, const void* x, int32_t M, int32_t stochastic, double* omega,
                                  void* hip_stream)
{
    if (!w_fp16 || !x || !omega) return LPQ_ERR_NULL;
    if (K < 128 || K % 128 != 0 || N < 1 || M < 1) return LPQ_ERR_SHAPE;
    if (misaligned(w_fp16) || misaligned(x) || (reinterpret_cast<uintptr_t>(omega) & 7u)) return LPQ_ERR_ALIGN;
    float* ws = nullptr;
    lpq_status st = workspace(false, indicator_workspace_bytes(N, (long)M * K / 8), &ws);
    if (st != LPQ_OK) return st;
    return launch_indicator(w_fp16, K, N, x, M, stochastic != 0, omega, ws, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? LPQ_OK : LPQ_ERR_DEVICE;
}

lpq_status lpq_unpack_dequant(const lpq_qweight* w, void* w_fp32, void* hip_stream)
{
    lpq_status st = check_weight(w);
    if (st != LPQ_OK) return st;
    if (!w_fp32) return LPQ_ERR_NULL;
    if (misaligned(w_fp32)) return LPQ_ERR_ALIGN;
    return launch_unpack_dequant(*w, static_cast<float*>(w_fp32), static_cast<hipStream_t>(hip_stream)) == hipSuccess ? LPQ_OK
                                                                                                                       : LPQ_ERR_DEVICE;
}

lpq_status lpq_qlinear_prefill(const lpq_qweight* w, const void* x, int32_t M, void* y, void* hip_stream)
{
    lpq_status st = check_linear(w, x, M, y);
    if (st != LPQ_OK) return st;
    std::vector<LinearCall> calls(1, LinearCall{w, x, y, nullptr, LPQ_ACT_NONE});
    return run_prefill(calls, M, static_cast<hipStream_t>(hip_stream));
}

lpq_status lpq_qlinear_decode(const lpq_qweight* w, const void* x, int32_t M, void* y, void* hip_stream)
{
    lpq_status st = check_linear(w, x, M, y);
    if (st != LPQ_OK) return st;
    std::vector<LinearCall> calls(1, LinearCall{w, x, y, nullptr, LPQ_ACT_NONE});
    return run_decode(calls, M, static_cast<hipStream_t>(hip_stream));
}

lpq_status lpq_qlinear_fused(const lpq_qweight* w, const void* x, int32_t M, void* y, const lpq_epilogue* ep, lpq_phase phase,
                             void* hip_stream)
{
    lpq_status st = check_linear(w, x, M, y);
    if (st != LPQ_OK) return st;
    if (phase != LPQ_PREFILL && phase != LPQ_DECODE) return LPQ_ERR_UNSUPPORTED;
    LinearCall c{w, x, y, nullptr, LPQ_ACT_NONE};
    if (ep) {
        if (ep->activation != LPQ_ACT_NONE && ep->activation != LPQ_ACT_RELU && ep->activation != LPQ_ACT_GELU_TANH)
            return LPQ_ERR_UNSUPPORTED;
        if (ep->residual && misaligned(ep->residual)) return LPQ_ERR_ALIGN;
        c.residual = ep->residual;
        c.act = ep->activation;
    }
    std::vector<LinearCall> calls(1, c);
    return phase == LPQ_PREFILL ? run_prefill(calls, M, static_cast<hipStream_t>(hip_stream))
                                : run_decode(calls, M, static_cast<hipStream_t>(hip_stream));
}

static lpq_status stage_linears(const lpq_layer* layers, int32_t n_layers, lpq_phase phase, int32_t M, const lpq_layer_io* io,
                                void* hip_stream, bool static_ws)
{
    if (!layers || !io) return LPQ_ERR_NULL;
    if (n_layers < 1 || n_layers > 4096) return LPQ_ERR_SHAPE;
    if (phase != LPQ_PREFILL && phase != LPQ_DECODE) return LPQ_ERR_UNSUPPORTED;
    std::vector<LinearCall> calls;
    calls.reserve((size_t)n_layers * 4);
    for (int32_t i = 0; i < n_layers; ++i) {
        const lpq_qweight* w[4] = {&layers[i].qkv, &layers[i].out, &layers[i].fc1, &layers[i].fc2};
        const void* xs[4] = {io[i].x_qkv, io[i].x_out, io[i].x_fc1, io[i].x_fc2};
        void* ys[4] = {io[i].y_qkv, io[i].y_out, io[i].y_fc1, io[i].y_fc2};
        for (int j = 0; j < 4; ++j) {
            lpq_status st = check_linear(w[j], xs[j], M, ys[j]);
            if (st != LPQ_OK) return st;
            calls.push_back(LinearCall{w[j], xs[j], ys[j], nullptr, LPQ_ACT_NONE});
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return phase == LPQ_DECODE ? run_decode(calls, M, stream, static_ws) : run_prefill(calls, M, stream, static_ws);
}

lpq_status lpq_stage_linears(const lpq_layer* layers, int32_t n_layers, lpq_phase phase, int32_t M, const lpq_layer_io* io,
                             void* hip_stream)
{
    return stage_linears(layers, n_layers, phase, M, io, hip_stream, false);
}

lpq_status lpq_stage_linears_noalloc(const lpq_layer* layers, int32_t n_layers, lpq_phase phase, int32_t M, const lpq_layer_io* io,
                                     void* hip_stream)
{
    return stage_linears(layers, n_layers, phase, M, io, hip_stream, true);
}

lpq_status lpq_workspace_policy(size_t have_bytes, int32_t reserved, size_t need_bytes, size_t* alloc_bytes)
{
    if (!alloc_bytes) return LPQ_ERR_NULL;
    return workspace_policy(have_bytes, reserved != 0, need_bytes, alloc_bytes);
}

lpq_status lpq_workspace_reserve(size_t bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LPQ_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_ws.mu);
    if (g_ws.bytes[dev] < bytes) {
        lpq_status st = workspace_grow(dev, bytes);
        if (st != LPQ_OK) return st;
    }
    g_ws.reserved[dev] = true;
    return LPQ_OK;
}

size_t lpq_workspace_bytes(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    std::lock_guard<std::mutex> lock(g_ws.mu);
    return g_ws.bytes[dev];
}

lpq_status lpq_set_decode_routing(int32_t rows_max_mib, int32_t rows_tiles)
{
    if (rows_max_mib > 4096 || (rows_tiles > 0 && (rows_tiles < 2 || rows_tiles > 5))) return LPQ_ERR_SHAPE;
    g_rows_max_mb.store(rows_max_mib < 0 ? 192 : rows_max_mib);
    g_rows_tiles.store(rows_tiles < 0 ? 0 : rows_tiles);
    return LPQ_OK;
}

const char* lpq_status_str(lpq_status status)
{
    switch (status) {
    case LPQ_OK: return "ok";
    case LPQ_ERR_NULL: return "null pointer";
    case LPQ_ERR_BITS: return "bits must be 3, 4, 8 or 16";
    case LPQ_ERR_SCHEME: return "bits / scheme / group_size do not match";
    case LPQ_ERR_SHAPE: return "bad shape or size (K % 128, N % 64, M >= 1, descriptor mismatch, malformed plan or samples)";
    case LPQ_ERR_ALIGN: return "pointer not 16-byte aligned";
    case LPQ_ERR_BUFSIZE: return "buffer too small, or workspace allocation failed";
    case LPQ_ERR_DEVICE: return "HIP call failed";
    case LPQ_ERR_UNSUPPORTED: return "unsupported request";
    }
    return "unknown status";
}

}  // extern "C"
