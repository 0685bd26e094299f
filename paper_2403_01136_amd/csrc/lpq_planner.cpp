// The assigner's cost models and the bitwidth-transfer heuristic of LLM-PQ (arXiv 2403.01136, Sec. 4.1 and 4.3).
// Host code only: these entry points take host pointers, run on the calling thread and never touch a device.
//
//   memory cost model     Sec. 4.1: bytes of embeddings, of a decoder layer at a bitwidth, of a layer's KV cache
//   latency cost model    Sec. 4.1: per-phase linear regression of one decoder layer's time, least squares by
//                         Householder QR (columns scaled to unit length first: they span 1 .. v s^2)
//   objective             Sec. 4.3, Eq. (1) with the stage-time, send-time and memory constraints
//   adabits               the program without latency, exact: an inner table gives, for every window of layers and
//                         every count of layers per bitwidth, the least summed indicator; an outer pass over the
//                         stages picks windows and counts that fit each device
//   bitwidth transfer     Sec. 4.3, Algorithm 2
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <vector>

#include "../../include/lpq.h"

namespace {

constexpr double INF = std::numeric_limits<double>::infinity();
constexpr int MAX_BITS_CHOICES = 4;

// ---- latency regression ---------------------------------------------------------------------------------------

int n_coef(int phase) { return phase == LPQ_PREFILL ? 5 : 4; }

void features(int phase, double v, double len, double* f)
{
    if (phase == LPQ_PREFILL) {
        f[0] = 1.0, f[1] = v, f[2] = len, f[3] = v * len, f[4] = v * len * len;
    } else {
        f[0] = 1.0, f[1] = v, f[2] = v * len, f[3] = len;
    }
}

// min ||A c - y|| for A [n][m] (row-major, overwritten), m <= 5.  false if A is rank deficient.
bool least_squares(std::vector<double>& A, std::vector<double>& y, int n, int m, double* c)
{
    double colscale[5];
    for (int k = 0; k < m; ++k) {
        double ss = 0.0;
        for (int i = 0; i < n; ++i) ss += A[(size_t)i * m + k] * A[(size_t)i * m + k];
        if (!(ss > 0.0)) return false;
        colscale[k] = 1.0 / std::sqrt(ss);
        for (int i = 0; i < n; ++i) A[(size_t)i * m + k] *= colscale[k];
    }
    for (int k = 0; k < m; ++k) {              // Householder reflection that zeroes column k below the diagonal
        double norm = 0.0;
        for (int i = k; i < n; ++i) norm += A[(size_t)i * m + k] * A[(size_t)i * m + k];
        norm = std::sqrt(norm);
        if (norm < 1e-11) return false;         // columns have unit length: this one lies in the span of the others
        const double alpha = A[(size_t)k * m + k] > 0 ? -norm : norm;
        std::vector<double> u(n - k);
        for (int i = k; i < n; ++i) u[i - k] = A[(size_t)i * m + k];
        u[0] -= alpha;
        double uu = 0.0;
        for (double e : u) uu += e * e;
        if (uu > 0.0) {
            for (int col = k; col < m; ++col) {
                double dot = 0.0;
                for (int i = k; i < n; ++i) dot += u[i - k] * A[(size_t)i * m + col];
                const double f = 2.0 * dot / uu;
                for (int i = k; i < n; ++i) A[(size_t)i * m + col] -= f * u[i - k];
            }
            double dot = 0.0;
            for (int i = k; i < n; ++i) dot += u[i - k] * y[i];
            const double f = 2.0 * dot / uu;
            for (int i = k; i < n; ++i) y[i] -= f * u[i - k];
        }
    }
    for (int k = m - 1; k >= 0; --k) {          // back substitution in R
        double acc = y[k];
        for (int col = k + 1; col < m; ++col) acc -= A[(size_t)k * m + col] * c[col];
        c[k] = acc / A[(size_t)k * m + k];
    }
    for (int k = 0; k < m; ++k) c[k] *= colscale[k];
    return true;
}

// ---- plans -----------------------------------------------------------------------------------------------------------

bool problem_ok(const lpq_plan_problem* p)
{
    return p && p->bits && p->omega && p->lat_pre && p->lat_dec && p->mem && p->cap;
}

bool sizes_ok(const lpq_plan_problem* p)
{
    if (!(p->L >= 1 && p->N >= 1 && p->N <= p->L && p->n_bits >= 1 && p->n_bits <= 64 && p->B >= 1 && p->eta >= 1 && p->xi >= 1 &&
          p->n >= 1))
        return false;
    for (int k = 0; k < p->n_bits; ++k)
        if (p->bits[k] < 1) return false;
    return true;
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

bool plan_well_formed(const lpq_plan_problem* p, const int32_t* counts, const int32_t* choice)
{
    long total = 0;
    for (int j = 0; j < p->N; ++j) {
        if (counts[j] < 1) return false;
        total += counts[j];
    }
    if (total != p->L) return false;
    for (int i = 0; i < p->L; ++i)
        if (choice[i] < 0 || choice[i] >= p->n_bits) return false;
    return true;
}

void stage_times(const lpq_plan_problem* p, const int32_t* counts, const int32_t* choice, std::vector<double>& tp, std::vector<double>& td)
{
    tp.assign(p->N, 0.0);
    td.assign(p->N, 0.0);
    int i = 0;
    for (int j = 0; j < p->N; ++j)
        for (int e = 0; e < counts[j]; ++e, ++i) {
            tp[j] += p->lat_pre[(size_t)j * p->n_bits + choice[i]];
            td[j] += p->lat_dec[(size_t)j * p->n_bits + choice[i]];
        }
}

// Eq. (1).  Sums run left to right over layers and stages.
double objective(const lpq_plan_problem* p, const int32_t* counts, const int32_t* choice, bool with_latency)
{
    if (!plan_well_formed(p, counts, choice)) return INF;
    int i = 0;
    for (int j = 0; j < p->N; ++j) {
        double need = 0.0;
        for (int e = 0; e < counts[j]; ++e, ++i) need += p->mem[choice[i]];
        if (j == 0) need += p->emb;
        if (need > p->cap[j]) return INF;
    }
    double q = 0.0;
    for (int l = 0; l < p->L; ++l) q += p->omega[(size_t)l * p->n_bits + choice[l]];
    const double quality = p->theta * q;
    if (!with_latency) return quality;
    std::vector<double> tp, td;
    stage_times(p, counts, choice, tp, td);
    double tmax_pre = 0.0, tmax_dec = 0.0, t_pre = 0.0, t_dec = 0.0;
    for (int j = 0; j < p->N; ++j) {
        tmax_pre = std::max(tmax_pre, std::max(tp[j], p->comm_pre ? p->comm_pre[j] : 0.0));
        tmax_dec = std::max(tmax_dec, std::max(td[j], p->comm_dec ? p->comm_dec[j] : 0.0));
        t_pre += tp[j];
        t_dec += td[j];
    }
    const int mu_pre = ceil_div(p->B, p->eta), mu_dec = ceil_div(p->B, p->xi);
    const double lat = (mu_pre - 1) * tmax_pre + (double)((mu_dec - 1) * (p->n - 1)) * tmax_dec + t_pre + t_dec;
    return lat + quality;
}

// Least summed indicator over all ways to give `cnt[k]` layers of the window [first, first + n) bitwidth k
// (n = sum of cnt).  Table over prefix counts in mixed radix; choice_out (may be null) receives one best assignment.
double assign_window(const lpq_plan_problem* p, int first, const int* cnt, int32_t* choice_out)
{
    const int nb = p->n_bits;
    std::vector<int> radix(nb), stride(nb);
    size_t states = 1;
    for (int k = 0; k < nb; ++k) {
        radix[k] = cnt[k] + 1;
        stride[k] = (int)states;
        states *= (size_t)radix[k];
    }
    std::vector<double> best(states, INF);
    std::vector<int8_t> from(states, -1);
    std::vector<int> digit(nb, 0);
    best[0] = 0.0;
    for (size_t s = 1; s < states; ++s) {
        for (int k = 0; k < nb; ++k) {            // increment the mixed-radix counter
            if (++digit[k] < radix[k]) break;
            digit[k] = 0;
        }
        int placed = 0;
        for (int k = 0; k < nb; ++k) placed += digit[k];
        const double* w = p->omega + (size_t)(first + placed - 1) * nb;   // the layer this state's last step placed
        for (int k = 0; k < nb; ++k) {
            if (digit[k] == 0) continue;
            const double v = best[s - stride[k]] + w[k];
            if (v < best[s]) best[s] = v, from[s] = (int8_t)k;
        }
    }
    if (choice_out) {
        size_t s = states - 1;
        int n = 0;
        for (int k = 0; k < nb; ++k) n += cnt[k];
        for (int l = n - 1; l >= 0; --l) {
            const int k = from[s];
            choice_out[l] = k;
            s -= stride[k];
        }
    }
    return best[states - 1];
}

struct Plan {
    std::vector<int32_t> counts;                  // layers per stage
    std::vector<std::vector<int>> cnt;            // per stage: layers per bitwidth
    std::vector<int32_t> choice;                  // per layer, derived: each stage's least-loss assignment
};

void derive_choice(const lpq_plan_problem* p, Plan& plan)
{
    plan.choice.assign(p->L, 0);
    int first = 0;
    for (int j = 0; j < p->N; ++j) {
        assign_window(p, first, plan.cnt[j].data(), plan.choice.data() + first);
        first += plan.counts[j];
    }
}

}  // namespace

extern "C" {

double lpq_mem_embedding_bytes(const lpq_model_shape* m)
{
    if (!m || m->h1 < 1 || m->vocab < 1 || m->d_t < 1 || m->pos < 0) return -1.0;
    const double proj = m->h1 != m->d_t ? 2.0 * (double)m->h1 * (double)m->d_t : 0.0;
    return ((double)m->vocab * m->d_t + (double)m->pos * m->d_t + proj + (double)m->vocab * m->d_t) * 2.0;
}

double lpq_mem_layer_bytes(const lpq_model_shape* m, int32_t bit)
{
    if (!m || m->h1 < 1 || m->h2 < 1 || bit < 1 || bit > 32) return -1.0;
    const double weights = 4.0 * (double)m->h1 * m->h1 + 2.0 * (double)m->h1 * m->h2;
    return weights * bit / 8.0 + (m->rmsnorm ? 4.0 : 6.0) * (double)m->h1;
}

double lpq_mem_kv_bytes(const lpq_model_shape* m, int64_t v, int64_t s, int64_t n, int32_t bit_kv)
{
    if (!m || m->h1 < 1 || v < 0 || s < 0 || n < 0 || bit_kv < 1 || bit_kv > 32) return -1.0;
    return 2.0 * (double)v * (double)(s + n) * (double)m->h1 * bit_kv / 8.0;
}

lpq_status lpq_latency_fit(lpq_phase phase, int32_t n_samples, const double* v, const double* len, const double* t, double* coef)
{
    if (!v || !len || !t || !coef) return LPQ_ERR_NULL;
    if (phase != LPQ_PREFILL && phase != LPQ_DECODE) return LPQ_ERR_UNSUPPORTED;
    const int m = n_coef(phase);
    if (n_samples < m) return LPQ_ERR_SHAPE;
    std::vector<double> A((size_t)n_samples * m), y(t, t + n_samples);
    for (int i = 0; i < n_samples; ++i) features(phase, v[i], len[i], &A[(size_t)i * m]);
    return least_squares(A, y, n_samples, m, coef) ? LPQ_OK : LPQ_ERR_SHAPE;
}

lpq_status lpq_latency_predict(lpq_phase phase, const double* coef, int32_t n, const double* v, const double* len, double* t_out)
{
    if (!coef || !v || !len || !t_out) return LPQ_ERR_NULL;
    if (phase != LPQ_PREFILL && phase != LPQ_DECODE) return LPQ_ERR_UNSUPPORTED;
    if (n < 0) return LPQ_ERR_SHAPE;
    const int m = n_coef(phase);
    for (int i = 0; i < n; ++i) {
        double f[5], acc = 0.0;
        features(phase, v[i], len[i], f);
        for (int k = 0; k < m; ++k) acc += f[k] * coef[k];
        t_out[i] = acc;
    }
    return LPQ_OK;
}

lpq_status lpq_plan_objective(const lpq_plan_problem* p, const int32_t* counts, const int32_t* choice, int32_t with_latency, double* obj)
{
    if (!problem_ok(p) || !counts || !choice || !obj) return LPQ_ERR_NULL;
    if (!sizes_ok(p)) return LPQ_ERR_SHAPE;
    *obj = objective(p, counts, choice, with_latency != 0);
    return LPQ_OK;
}

lpq_status lpq_plan_adabits(const lpq_plan_problem* p, int32_t* counts, int32_t* choice, double* obj)
{
    if (!problem_ok(p) || !counts || !choice || !obj) return LPQ_ERR_NULL;
    if (!sizes_ok(p) || p->n_bits > MAX_BITS_CHOICES) return LPQ_ERR_SHAPE;
    const int L = p->L, N = p->N, nb = p->n_bits;
    const int max_len = L - N + 1;                           // every other stage keeps one layer
    // window_best[j][a][len]: least summed indicator of layers [a, a + len) on device j within its memory
    const size_t per_dev = (size_t)L * (max_len + 1);
    std::vector<double> window_best((size_t)N * per_dev, INF);
    // level tables over the counts of the first nb - 1 bitwidths (the last follows from the level)
    size_t cells = 1;
    for (int k = 0; k + 1 < nb; ++k) cells *= (size_t)(max_len + 1);
    if (cells * sizeof(double) * 2 > ((size_t)1 << 30)) return LPQ_ERR_BUFSIZE;
    std::vector<double> cur(cells), nxt(cells);
    std::vector<int> c(nb);
    auto for_each_cell = [&](int level, auto&& fn) {         // every count vector with sum == level
        // enumerate c[0..nb-2] with partial sums <= level; c[nb-1] = level - sum
        std::fill(c.begin(), c.end(), 0);
        while (true) {
            int sum = 0;
            size_t idx = 0, mul = 1;
            for (int k = 0; k + 1 < nb; ++k) sum += c[k], idx += mul * c[k], mul *= (size_t)(max_len + 1);
            if (sum <= level) {
                c[nb - 1] = level - sum;
                fn(idx);
            }
            int k = 0;
            for (; k + 1 < nb; ++k) {
                if (++c[k] <= level) break;
                c[k] = 0;
            }
            if (k + 1 >= nb) break;
        }
    };
    std::vector<size_t> stride(nb, 0);
    {
        size_t mul = 1;
        for (int k = 0; k + 1 < nb; ++k) stride[k] = mul, mul *= (size_t)(max_len + 1);
    }
    for (int a = 0; a < L; ++a) {
        std::fill(cur.begin(), cur.end(), INF);
        cur[0] = 0.0;
        const int lim = std::min(max_len, L - a);
        for (int len = 1; len <= lim; ++len) {
            std::fill(nxt.begin(), nxt.end(), INF);
            const double* w = p->omega + (size_t)(a + len - 1) * nb;
            for_each_cell(len, [&](size_t idx) {
                double best = INF;
                for (int k = 0; k < nb; ++k) {
                    if (c[k] == 0) continue;
                    const double prev = cur[idx - stride[k]];      // stride of the last bitwidth is 0: same cell index
                    if (prev + w[k] < best) best = prev + w[k];
                }
                nxt[idx] = best;
                if (best == INF) return;
                double need = 0.0;
                for (int k = 0; k < nb; ++k) need += c[k] * p->mem[k];
                for (int j = 0; j < N; ++j)
                    if (need + (j == 0 ? p->emb : 0.0) <= p->cap[j]) {
                        double& slot = window_best[(size_t)j * per_dev + (size_t)a * (max_len + 1) + len];
                        if (best < slot) slot = best;
                    }
            });
            cur.swap(nxt);
        }
    }
    // stages: f[j][i] = least sum for layers [0, i) on devices 0..j
    std::vector<double> f((size_t)N * (L + 1), INF);
    std::vector<int> cut((size_t)N * (L + 1), -1);
    for (int i = 1; i <= std::min(L, max_len); ++i) f[i] = window_best[(size_t)0 * (max_len + 1) + i], cut[i] = 0;
    for (int j = 1; j < N; ++j)
        for (int i = j + 1; i <= L; ++i)
            for (int a = j; a < i; ++a) {
                if (i - a > max_len || f[(size_t)(j - 1) * (L + 1) + a] == INF) continue;
                const double wv = window_best[(size_t)j * per_dev + (size_t)a * (max_len + 1) + (i - a)];
                if (wv == INF) continue;
                const double v = f[(size_t)(j - 1) * (L + 1) + a] + wv;
                if (v < f[(size_t)j * (L + 1) + i]) f[(size_t)j * (L + 1) + i] = v, cut[(size_t)j * (L + 1) + i] = a;
            }
    if (f[(size_t)(N - 1) * (L + 1) + L] == INF) {
        *obj = INF;
        return LPQ_OK;
    }
    std::vector<int> start(N + 1);
    start[N] = L;
    for (int j = N - 1; j >= 0; --j) start[j] = cut[(size_t)j * (L + 1) + start[j + 1]];
    // per stage: the feasible count vector that attains the window's value, then its assignment
    for (int j = 0; j < N; ++j) {
        const int a = start[j], len = start[j + 1] - a;
        counts[j] = len;
        std::vector<int> cnt(nb, 0), best_cnt(nb, 0);
        double best = INF;
        // enumerate count vectors of this window directly (len is small next to the tables above)
        std::vector<int> cc(nb, 0);
        while (true) {
            int sum = 0;
            for (int k = 0; k + 1 < nb; ++k) sum += cc[k];
            if (sum <= len) {
                cc[nb - 1] = len - sum;
                double need = 0.0;
                for (int k = 0; k < nb; ++k) need += cc[k] * p->mem[k];
                if (need + (j == 0 ? p->emb : 0.0) <= p->cap[j]) {
                    const double v = assign_window(p, a, cc.data(), nullptr);
                    if (v < best) best = v, best_cnt = cc;
                }
            }
            int k = 0;
            for (; k + 1 < nb; ++k) {
                if (++cc[k] <= len) break;
                cc[k] = 0;
            }
            if (k + 1 >= nb) break;
        }
        assign_window(p, a, best_cnt.data(), choice + a);
    }
    *obj = objective(p, counts, choice, false);
    return LPQ_OK;
}

lpq_status lpq_plan_bitwidth_transfer(const lpq_plan_problem* p, int32_t* counts, int32_t* choice, double* obj, int32_t* rounds)
{
    if (!problem_ok(p) || !counts || !choice || !obj || !rounds) return LPQ_ERR_NULL;
    if (!sizes_ok(p) || !plan_well_formed(p, counts, choice)) return LPQ_ERR_SHAPE;
    const int N = p->N, nb = p->n_bits;
    Plan plan;
    plan.counts.assign(counts, counts + N);
    plan.cnt.assign(N, std::vector<int>(nb, 0));
    {
        int i = 0;
        for (int j = 0; j < N; ++j)
            for (int e = 0; e < counts[j]; ++e, ++i) plan.cnt[j][choice[i]]++;
    }
    derive_choice(p, plan);
    double obj0 = objective(p, plan.counts.data(), plan.choice.data(), true);
    const int mu_pre = ceil_div(p->B, p->eta), mu_dec = ceil_div(p->B, p->xi);
    const double w_pre = (double)mu_pre, w_dec = (double)((mu_dec - 1) * (p->n - 1) + 1);
    int applied = 0;
    std::vector<double> tp, td;
    while (true) {
        stage_times(p, plan.counts.data(), plan.choice.data(), tp, td);
        std::vector<int> order(N);
        std::vector<double> key(N);
        for (int j = 0; j < N; ++j) order[j] = j, key[j] = w_pre * tp[j] + w_dec * td[j];
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return key[x] < key[y]; });
        const int st = order[N - 1];
        bool found = false;
        Plan sol;
        for (int o = 0; o + 1 < N; ++o) {
            const int pi = order[o];
            for (int ia = 0; ia < nb; ++ia)
                for (int ib = 0; ib < nb; ++ib) {
                    if (p->bits[ia] == p->bits[ib]) continue;
                    const int nums = std::max(1, p->bits[ib] / p->bits[ia]);
                    if (plan.cnt[st][ia] < nums || plan.cnt[pi][ib] < 1) continue;
                    Plan cand;
                    cand.counts = plan.counts;
                    cand.cnt = plan.cnt;
                    cand.cnt[st][ia] -= nums, cand.cnt[pi][ia] += nums;
                    cand.cnt[pi][ib] -= 1, cand.cnt[st][ib] += 1;
                    cand.counts[st] += 1 - nums, cand.counts[pi] += nums - 1;
                    derive_choice(p, cand);
                    const double v = objective(p, cand.counts.data(), cand.choice.data(), true);
                    if (v < obj0) obj0 = v, sol = std::move(cand), found = true;
                }
        }
        if (!found) break;
        plan = std::move(sol);
        ++applied;
    }
    std::memcpy(counts, plan.counts.data(), sizeof(int32_t) * N);
    std::memcpy(choice, plan.choice.data(), sizeof(int32_t) * p->L);
    *obj = obj0;
    *rounds = applied;
    return LPQ_OK;
}

}  // extern "C"
