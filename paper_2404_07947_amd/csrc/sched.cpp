// Schedule simulator (Section 6) and branch-and-bound scheduling (Section 5, Algorithm 1): host code behind
// include/exe_sched.h.  Nothing here touches the GPU.
#include "../../include/exe_sched.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <map>
#include <queue>
#include <vector>

namespace exe {
int set_error(int code, const char* msg);      // runtime.hip: stores the message exe_last_error() returns
}

namespace {

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    return exe::set_error(code, buf);
}

// entry s-1 = probability of length s
struct Dist {
    const double* p;
    int n;
    double mean() const
    {
        double m = 0;
        for (int s = 1; s <= n; ++s) m += s * p[s - 1];
        return m;
    }
    double second() const
    {
        double m = 0;
        for (int s = 1; s <= n; ++s) m += (double)s * s * p[s - 1];
        return m;
    }
};

int check_dist(const double* p, int n, const char* what)
{
    if (!p || n < 1) return fail(EXE_ERR_ARG, "%s: empty distribution", what);
    double sum = 0;
    for (int i = 0; i < n; ++i) {
        if (!(p[i] >= 0.0)) return fail(EXE_ERR_ARG, "%s: negative or NaN probability at length %d", what, i + 1);
        sum += p[i];
    }
    if (fabs(sum - 1.0) > 1e-6) return fail(EXE_ERR_ARG, "%s: probabilities sum to %.9g, not 1", what, sum);
    return EXE_OK;
}

// P_D(U), U = 1..n_d: every output length S contributes its whole mass (S <= N_D) or the share 1 / ceil(S / N_D)
// of it (S > N_D) to the one iteration at which its last token is produced
void completion(const Dist& out, int n_d, std::vector<double>& p_u)
{
    p_u.assign(n_d, 0.0);
    for (int s = 1; s <= out.n; ++s) {
        double mass = out.p[s - 1];
        if (mass == 0.0) continue;
        if (s <= n_d) {
            p_u[s - 1] += mass;
        } else {
            int phases = (s + n_d - 1) / n_d;
            p_u[(s - 1) % n_d] += mass / phases;
        }
    }
}

// one phase's step times on its (batch x length) grid
struct Grid {
    std::vector<int> batches, lengths;
    std::vector<double> ms;      // [batches][lengths]
    double at(int i, int j) const { return ms[(size_t)i * lengths.size() + j]; }
};

int build_grid(const exe_sim_table_t* t, int phase, Grid& g)
{
    if (!t || !t->rows || t->n_rows < 1) return fail(EXE_ERR_ARG, "empty profile table");
    int layers = phase == 0 ? t->n_layers_encode : t->n_layers_decode;
    if (layers < 1) return fail(EXE_ERR_ARG, "layer count of phase %d must be positive", phase);
    std::map<std::pair<int, int>, double> cell;
    for (int i = 0; i < t->n_rows; ++i) {
        const exe_profile_row_t& r = t->rows[i];
        if (r.phase != phase) continue;
        if (r.batch < 1 || r.length < 1) return fail(EXE_ERR_ARG, "profile row %d: batch and length must be positive", i);
        cell[{r.batch, r.length}] = layers * ((double)r.attn_ms_per_layer + (double)r.rest_ms_per_layer) + (double)r.head_ms;
        g.batches.push_back(r.batch);
        g.lengths.push_back(r.length);
    }
    if (cell.empty()) return fail(EXE_ERR_ARG, "profile table has no row of phase %d", phase);
    auto uniq = [](std::vector<int>& v) {
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
    };
    uniq(g.batches);
    uniq(g.lengths);
    if (cell.size() != g.batches.size() * g.lengths.size())
        return fail(EXE_ERR_ARG, "phase %d rows do not form a full batch x length grid (%zu of %zu cells)", phase,
                    cell.size(), g.batches.size() * g.lengths.size());
    g.ms.reserve(cell.size());
    for (int b : g.batches)
        for (int l : g.lengths) g.ms.push_back(cell[{b, l}]);
    return EXE_OK;
}

// index of the grid interval that holds x (x already clamped into the grid) and the position inside it
void locate(const std::vector<int>& grid, double x, int& lo, int& hi, double& f)
{
    if (grid.size() == 1) {
        lo = hi = 0;
        f = 0.0;
        return;
    }
    auto it = std::lower_bound(grid.begin() + 1, grid.end() - 1, x, [](int g, double v) { return g < v; });
    hi = (int)(it - grid.begin());
    lo = hi - 1;
    f = (x - grid[lo]) / (double)(grid[hi] - grid[lo]);
}

double step_ms(const Grid& g, double batch, double length)
{
    if (batch <= 0) return 0.0;
    double scale = 1.0, b = batch;
    double bmax = g.batches.back(), bmin = g.batches.front();
    if (b > bmax) {
        scale = b / bmax;
        b = bmax;
    }
    if (b < bmin) {
        scale = b / bmin;
        b = bmin;
    }
    double l = std::min(std::max(length, (double)g.lengths.front()), (double)g.lengths.back());
    int i0, i1, j0, j1;
    double fb, fl;
    locate(g.batches, b, i0, i1, fb);
    locate(g.lengths, l, j0, j1, fl);
    double low = (1 - fl) * g.at(i0, j0) + fl * g.at(i0, j1);
    double high = (1 - fl) * g.at(i1, j0) + fl * g.at(i1, j1);
    return ((1 - fb) * low + fb * high) * scale;
}

struct RraInputs {
    Grid enc, dec;
    Dist in, out;
    double mean_in, ctx, occupancy;
};

void simulate_rra(const RraInputs& x, double b_d, int n_d, int latency_len, exe_sim_rra_result_t& r)
{
    std::vector<double> p_u;
    completion(x.out, n_d, p_u);
    double frac = 0;
    for (double v : p_u) frac += v;
    r.b_d = b_d;
    r.completed_fraction = frac;
    r.b_e = b_d * frac;
    r.context_length = x.ctx;
    r.encode_ms = step_ms(x.enc, r.b_e, x.mean_in);
    int phases = (latency_len + n_d - 1) / n_d, last = 1 + (latency_len - 1) % n_d;
    double done = 0, dec = 0, tokens = 0, head = 0;
    for (int u = 1; u <= n_d; ++u) {
        double live = b_d * (1.0 - done);
        double t = step_ms(x.dec, live, x.ctx);
        dec += t;
        tokens += live;
        if (u <= last) head += t;
        done += p_u[u - 1];
    }
    r.decode_ms = dec;
    r.cycle_ms = r.encode_ms + dec;
    r.tokens_per_cycle = tokens;
    r.throughput_tok_s = tokens / r.cycle_ms * 1e3;
    r.throughput_seq_s = r.b_e / r.cycle_ms * 1e3;
    r.latency_ms = r.encode_ms + (phases - 1) * r.cycle_ms + head;
    double occ = 0;
    for (int s = 1; s <= x.out.n; ++s) occ += (double)((s + n_d - 1) / n_d) * x.out.p[s - 1];
    r.occupancy_exact = occ;
}

int prepare_rra(const exe_sim_table_t* table, const double* p_in, int in_max, const double* p_out, int out_max,
                RraInputs& x)
{
    int rc;
    if ((rc = check_dist(p_in, in_max, "input lengths")) != EXE_OK) return rc;
    if ((rc = check_dist(p_out, out_max, "output lengths")) != EXE_OK) return rc;
    if ((rc = build_grid(table, 0, x.enc)) != EXE_OK) return rc;
    if ((rc = build_grid(table, 1, x.dec)) != EXE_OK) return rc;
    x.in = Dist{p_in, in_max};
    x.out = Dist{p_out, out_max};
    x.mean_in = x.in.mean();
    x.ctx = x.mean_in + x.out.second() / (2.0 * x.out.mean()) + 0.5;
    return EXE_OK;
}

// ---------------------------------------------------------------- Algorithm 1
struct Point { double latency, throughput; };
struct Block {
    int lo1, lo2, hi1, hi2;
    double lower_thr, upper_thr;
    bool alive;
};

}  // namespace

extern "C" int exe_sim_completion(const double* p_out, int32_t s_max, int32_t n_decode, double* p_u,
                                  double* completed_fraction)
{
    if (!p_u || n_decode < 1) return fail(EXE_ERR_ARG, "n_decode must be positive and p_u non-null");
    int rc = check_dist(p_out, s_max, "output lengths");
    if (rc != EXE_OK) return rc;
    std::vector<double> v;
    completion(Dist{p_out, s_max}, n_decode, v);
    double sum = 0;
    for (int u = 0; u < n_decode; ++u) sum += (p_u[u] = v[u]);
    if (completed_fraction) *completed_fraction = sum;
    return EXE_OK;
}

extern "C" int exe_sim_step_ms(const exe_sim_table_t* table, int32_t phase, double batch, double length, double* ms)
{
    if (!ms || (phase != 0 && phase != 1)) return fail(EXE_ERR_ARG, "phase must be 0 or 1 and ms non-null");
    Grid g;
    int rc = build_grid(table, phase, g);
    if (rc != EXE_OK) return rc;
    *ms = step_ms(g, batch, length);
    return EXE_OK;
}

extern "C" int exe_sim_rra(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out,
                           int32_t out_max, double decode_batch, int32_t n_decode, int32_t latency_len,
                           exe_sim_rra_result_t* result)
{
    if (!result || !(decode_batch > 0) || n_decode < 1 || latency_len < 1)
        return fail(EXE_ERR_ARG, "decode_batch, n_decode and latency_len must be positive and result non-null");
    RraInputs x;
    int rc = prepare_rra(table, p_in, in_max, p_out, out_max, x);
    if (rc != EXE_OK) return rc;
    simulate_rra(x, decode_batch, n_decode, latency_len, *result);
    return EXE_OK;
}

extern "C" int exe_sim_waa(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out,
                           int32_t out_max, double encode_batch, int32_t n_gpus, exe_sim_waa_result_t* result)
{
    if (!result || !(encode_batch > 0) || n_gpus < 1)
        return fail(EXE_ERR_ARG, "encode_batch and n_gpus must be positive and result non-null");
    RraInputs x;
    int rc = prepare_rra(table, p_in, in_max, p_out, out_max, x);
    if (rc != EXE_OK) return rc;
    exe_sim_waa_result_t r;
    r.b_e = encode_batch;
    r.b_d = encode_batch * x.out.mean();
    r.encode_ms = step_ms(x.enc, r.b_e, x.mean_in);
    r.decode_ms = step_ms(x.dec, r.b_d, x.ctx);
    if (n_gpus >= 2) {
        long ge = lround(n_gpus * r.encode_ms / (r.encode_ms + r.decode_ms));
        r.gpus_encode = (int32_t)std::min<long>(std::max<long>(ge, 1), n_gpus - 1);
        r.gpus_decode = n_gpus - r.gpus_encode;
    } else {
        r.gpus_encode = r.gpus_decode = 1;
    }
    double period = std::max(r.encode_ms / r.gpus_encode, r.decode_ms / r.gpus_decode);
    r.throughput_seq_s = r.b_e / period * 1e3;
    *result = r;
    return EXE_OK;
}

extern "C" int exe_sched_search(exe_perf_fn perf, void* user, int32_t a1, int32_t b1, int32_t a2, int32_t b2,
                                double eps_throughput, double eps_latency, double latency_bound,
                                exe_sched_result_t* result)
{
    if (!perf || !result) return fail(EXE_ERR_ARG, "null perf or result");
    if (a1 > b1 || a2 > b2) return fail(EXE_ERR_ARG, "empty range");
    if ((int64_t)(b1 - a1 + 1) * (b2 - a2 + 1) > (int64_t)1 << 40) return fail(EXE_ERR_ARG, "range too large");
    std::map<std::pair<int, int>, Point> seen;
    int status = EXE_OK;
    auto eval = [&](int x1, int x2) -> Point {
        auto key = std::make_pair(x1, x2);
        auto it = seen.find(key);
        if (it != seen.end()) return it->second;
        Point p{0, 0};
        if (status == EXE_OK && perf(x1, x2, user, &p.latency, &p.throughput) != 0)
            status = fail(EXE_ERR_ARG, "perf failed at (%d, %d)", x1, x2);
        seen[key] = p;
        return p;
    };
    exe_sched_result_t r{};
    auto take = [&](const Point& p, int x1, int x2) {       // a point that meets the bound and beats T*
        r.found = 1;
        r.x1 = x1;
        r.x2 = x2;
        r.throughput = p.throughput;
        r.latency = p.latency;
    };
    Point low = eval(a1, a2), top = eval(b1, b2);
    if (status != EXE_OK) return status;
    if (low.latency < latency_bound) take(low, a1, a2);
    if (top.latency < latency_bound) {                      // the bound holds at the far corner: it is the optimum
        take(top, b1, b2);
        r.evaluations = (int32_t)seen.size();
        *result = r;
        return EXE_OK;
    }
    std::vector<Block> blocks;
    auto by_lower = [&](int x, int y) { return blocks[x].lower_thr < blocks[y].lower_thr; };
    std::priority_queue<int, std::vector<int>, decltype(by_lower)> queue(by_lower);
    blocks.push_back(Block{a1, a2, b1, b2, low.throughput, top.throughput, true});
    queue.push(0);
    while (!queue.empty() && status == EXE_OK) {
        int id = queue.top();
        queue.pop();
        if (!blocks[id].alive) continue;
        blocks[id].alive = false;
        Block B = blocks[id];
        ++r.blocks;
        int w1 = B.hi1 - B.lo1, w2 = B.hi2 - B.lo2;
        if (w1 == 0 && w2 == 0) continue;
        // splitting heuristic: towards the corner (top left or bottom right) with the higher throughput within the bound
        Point tl = eval(B.lo1, B.hi2), br = eval(B.hi1, B.lo2);
        bool tl_ok = tl.latency < latency_bound, br_ok = br.latency < latency_bound;
        bool cut_x1;
        if (tl_ok && (!br_ok || tl.throughput >= br.throughput)) cut_x1 = true;
        else if (br_ok) cut_x1 = false;
        else cut_x1 = w1 >= w2;
        if (cut_x1 && w1 == 0) cut_x1 = false;
        if (!cut_x1 && w2 == 0) cut_x1 = true;
        Block child[2];
        if (cut_x1) {
            int mid = B.lo1 + w1 / 2;
            child[0] = Block{B.lo1, B.lo2, mid, B.hi2, 0, 0, true};
            child[1] = Block{mid + 1, B.lo2, B.hi1, B.hi2, 0, 0, true};
        } else {
            int mid = B.lo2 + w2 / 2;
            child[0] = Block{B.lo1, B.lo2, B.hi1, mid, 0, 0, true};
            child[1] = Block{B.lo1, mid + 1, B.hi1, B.hi2, 0, 0, true};
        }
        bool have = false;
        Point best_upp{0, 0};
        int bx1 = 0, bx2 = 0;
        for (Block& c : child) {
            Point upp = eval(c.hi1, c.hi2), lowr = eval(c.lo1, c.lo2);
            c.lower_thr = lowr.throughput;
            c.upper_thr = upp.throughput;
            if (lowr.latency < latency_bound + eps_latency) {
                blocks.push_back(c);
                queue.push((int)blocks.size() - 1);
            }
            if (upp.latency < latency_bound && (!have || upp.throughput > best_upp.throughput)) {
                have = true;
                best_upp = upp;
                bx1 = c.hi1;
                bx2 = c.hi2;
            }
        }
        if (have && (!r.found || best_upp.throughput > r.throughput)) take(best_upp, bx1, bx2);
        if (r.found)
            for (Block& q : blocks)
                if (q.alive && q.upper_thr + eps_throughput < r.throughput) q.alive = false;
    }
    if (status != EXE_OK) return status;
    r.evaluations = (int32_t)seen.size();
    *result = r;
    return EXE_OK;
}

namespace {
struct RraPerf {
    const RraInputs* x;
    int nd_max, latency_len;
};
int rra_perf(int32_t x1, int32_t x2, void* user, double* latency, double* throughput)
{
    const RraPerf* p = (const RraPerf*)user;
    exe_sim_rra_result_t r;
    simulate_rra(*p->x, (double)x1, p->nd_max - x2, p->latency_len, r);
    *latency = r.latency_ms;
    *throughput = r.throughput_tok_s;
    return 0;
}
}  // namespace

extern "C" int exe_sched_rra(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out,
                             int32_t out_max, int32_t bd_min, int32_t bd_max, int32_t nd_min, int32_t nd_max,
                             int32_t latency_len, double latency_bound_ms, double eps_throughput, double eps_latency_ms,
                             exe_sched_rra_result_t* result)
{
    if (!result || bd_min < 1 || bd_max < bd_min || nd_min < 1 || nd_max < nd_min || latency_len < 1)
        return fail(EXE_ERR_ARG, "ranges must be positive and ordered, latency_len positive, result non-null");
    RraInputs x;
    int rc = prepare_rra(table, p_in, in_max, p_out, out_max, x);
    if (rc != EXE_OK) return rc;
    RraPerf ctx{&x, nd_max, latency_len};
    exe_sched_rra_result_t out{};
    rc = exe_sched_search(rra_perf, &ctx, bd_min, bd_max, 0, nd_max - nd_min, eps_throughput, eps_latency_ms,
                          latency_bound_ms, &out.search);
    if (rc != EXE_OK) return rc;
    if (out.search.found) {
        out.decode_batch = out.search.x1;
        out.n_decode = nd_max - out.search.x2;
        simulate_rra(x, (double)out.decode_batch, out.n_decode, latency_len, out.sim);
    }
    *result = out;
    return EXE_OK;
}
