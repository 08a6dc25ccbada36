// Host-side ConfLayers policy: skip-set selection from per-layer confidences (Section 3.2,
// Eq. 5-10) and the interval-based periodic search (Section 3.3).  Pure C++ in double
// precision, no device code; compiled with -ffp-contract=off so every sum rounds the same
// way on every build.  Where the paper leaves a detail open, the reading taken is spelled out
// at the place it is used.
#include "../../include/ssd.h"

#include <algorithm>
#include <cmath>
#include <deque>
#include <set>
#include <string>
#include <vector>

namespace {

struct Selection {
    std::vector<int> cand;       // model indices of the candidate layers
    std::vector<double> margin;  // c_hat_i - (mu_local_i - lambda * sigma_local_i), per candidate
    std::vector<uint8_t> mask;   // per model layer
    int n_min = 0, n_max = 0;
};

void mean_std(const double* v, int n, double& mu, double& sd)
{
    mu = 0.0; sd = 0.0;
    if (n == 0) return;
    double s = 0.0;
    for (int i = 0; i < n; i++) s += v[i];
    mu = s / n;
    double q = 0.0;
    for (int i = 0; i < n; i++) q += (v[i] - mu) * (v[i] - mu);
    sd = std::sqrt(q / n);  // population standard deviation
}

// Discrete gradient with unit spacing: central differences inside, one-sided at both ends.
std::vector<double> gradient(const std::vector<double>& y)
{
    const int n = (int)y.size();
    std::vector<double> g(n, 0.0);
    if (n < 2) return g;
    g[0] = y[1] - y[0];
    g[n - 1] = y[n - 1] - y[n - 2];
    for (int i = 1; i + 1 < n; i++) g[i] = (y[i + 1] - y[i - 1]) / 2.0;
    return g;
}

bool valid_params(const ssd_select_params* p)
{
    return p && p->lambda >= 0.0 && p->w_base >= 0.0 && p->kappa >= 0.0 && p->flat_tol >= 0.0 && p->min_ratio >= 0.0 &&
           p->max_ratio <= 1.0 && p->min_ratio <= p->max_ratio && p->eps >= 0.0;
}

void candidates(int L, const ssd_select_params& p, std::vector<int>& cand)
{
    cand.clear();
    if (p.protect_ends) { for (int l = 1; l + 1 < L; l++) cand.push_back(l); }
    else { for (int l = 0; l < L; l++) cand.push_back(l); }
}

void ratio_bounds(int L, int n, const ssd_select_params& p, int& n_min, int& n_max)
{
    n_min = std::min(n, (int)std::ceil(p.min_ratio * L - 1e-9));
    n_max = std::min(n, (int)std::floor(p.max_ratio * L + 1e-9));
    n_min = std::min(n_min, n_max);
}

Selection select(const double* conf, int L, const ssd_select_params& p)
{
    Selection S;
    S.mask.assign(L, 0);
    candidates(L, p, S.cand);
    const int n = (int)S.cand.size();
    if (n == 0) return S;
    std::vector<double> c(n);
    for (int i = 0; i < n; i++) c[i] = conf[S.cand[i]];

    double mu, sigma;                                       // Eq. 5
    mean_std(c.data(), n, mu, sigma);
    std::vector<double> chat(n);
    for (int i = 0; i < n; i++) chat[i] = (c[i] - mu) / (sigma + p.eps);

    std::vector<double> g = gradient(gradient(chat));       // Eq. 6: second-order gradient, magnitude,
    for (double& v : g) v = std::fabs(v);                   // min-max rescaled to [0, 1]
    double gmin = *std::min_element(g.begin(), g.end()), gmax = *std::max_element(g.begin(), g.end());
    for (double& v : g) v = (v - gmin) / (gmax - gmin + p.eps);

    // w_max grows with the number of leading layers that share the first layer's confidence
    int n_flat = 0;
    for (int i = 0; i < n; i++) {
        if (std::fabs(c[i] - c[0]) <= p.flat_tol) n_flat++;
        else break;
    }
    const double w_max = p.fixed_w_max >= 0.0 ? p.fixed_w_max : p.kappa * n_flat;

    S.margin.assign(n, 0.0);
    std::vector<int> chosen;
    std::vector<double> nb;
    for (int i = 0; i < n; i++) {
        // Eq. 7, floored to an integer half-width; l_i is the model's own layer index
        const int w = (int)std::floor(p.w_base + w_max * g[i] * ((double)S.cand[i] / (double)L));
        nb.clear();
        for (int j = std::max(0, i - w); j < std::min(n, i + w + 1); j++)
            if (j != i) nb.push_back(chat[j]);
        double m_loc, s_loc;                                // Eq. 8, 9 (window excludes the layer itself)
        mean_std(nb.data(), (int)nb.size(), m_loc, s_loc);
        S.margin[i] = chat[i] - (m_loc - p.lambda * s_loc); // Eq. 10: skip iff negative
        if (S.margin[i] < 0.0) chosen.push_back(i);
    }

    ratio_bounds(L, n, p, S.n_min, S.n_max);
    std::vector<int> order(n);
    for (int i = 0; i < n; i++) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        return S.margin[a] < S.margin[b] || (S.margin[a] == S.margin[b] && a < b);
    });
    std::vector<uint8_t> in(n, 0);
    for (int i : chosen) in[i] = 1;
    int cnt = (int)chosen.size();
    if (cnt < S.n_min) {
        for (int i : order) {
            if (cnt >= S.n_min) break;
            if (!in[i]) { in[i] = 1; cnt++; }
        }
    } else if (cnt > S.n_max) {
        int kept = 0;
        for (int i : order) {
            if (!in[i]) continue;
            if (kept < S.n_max) kept++;
            else in[i] = 0;
        }
    }
    for (int i = 0; i < n; i++) S.mask[S.cand[i]] = in[i];
    return S;
}

void uniform(int L, const ssd_select_params& p, std::vector<uint8_t>& mask)
{
    std::vector<int> cand;
    candidates(L, p, cand);
    int n_min, n_max;
    ratio_bounds(L, (int)cand.size(), p, n_min, n_max);
    mask.assign(L, 0);
    int picked = 0;
    for (size_t i = 0; i < cand.size() && picked < n_max; i += 2) { mask[cand[i]] = 1; picked++; }
}

}  // namespace

struct ssd_search {
    int L;
    ssd_search_params sp;
    ssd_select_params sel;
    std::deque<std::vector<double>> ring;
    std::vector<uint8_t> mask, best_mask;
    double best_score;
    bool active;
    int rounds, iters;
    long acc;
    std::set<std::string> evaluated;
};

extern "C" {

void ssd_select_defaults(ssd_select_params* p)
{
    if (!p) return;
    p->lambda = 0.3; p->w_base = 2.0; p->kappa = 1.0; p->flat_tol = 1e-3; p->min_ratio = 0.40; p->max_ratio = 0.60;
    p->protect_ends = 1; p->eps = 1e-8; p->fixed_w_max = -1.0;
}

int ssd_select_skip(const double* conf, int n_layers, const ssd_select_params* p, uint8_t* mask_out,
                    int32_t* n_skipped_out, double* margin_out)
{
    if (!conf || n_layers < 0 || !mask_out || !valid_params(p)) return SSD_EINVAL;
    for (int l = 0; l < n_layers; l++)
        if (!std::isfinite(conf[l])) return SSD_EINVAL;
    Selection S = select(conf, n_layers, *p);
    int cnt = 0;
    for (int l = 0; l < n_layers; l++) { mask_out[l] = S.mask[l]; cnt += S.mask[l]; }
    if (n_skipped_out) *n_skipped_out = cnt;
    if (margin_out) {
        for (int l = 0; l < n_layers; l++) margin_out[l] = 0.0;
        for (size_t i = 0; i < S.cand.size(); i++) margin_out[S.cand[i]] = S.margin[i];
    }
    return SSD_OK;
}

int ssd_uniform_skip(int n_layers, const ssd_select_params* p, uint8_t* mask_out)
{
    if (n_layers < 0 || !mask_out || !valid_params(p)) return SSD_EINVAL;
    std::vector<uint8_t> m;
    uniform(n_layers, *p, m);
    for (int l = 0; l < n_layers; l++) mask_out[l] = m[l];
    return SSD_OK;
}

void ssd_search_defaults(ssd_search_params* p)
{
    if (!p) return;
    p->opt_interval = 30; p->score_goal = 4.0; p->max_rounds = 10; p->window = 100;
}

int ssd_search_create(int n_layers, const ssd_search_params* sp, const ssd_select_params* sel, ssd_search** out)
{
    if (!out) return SSD_EINVAL;
    *out = nullptr;
    if (n_layers < 1 || !sp || !valid_params(sel) || sp->opt_interval < 1 || sp->max_rounds < 1 || sp->window < 1)
        return SSD_EINVAL;
    ssd_search* s = new ssd_search();
    s->L = n_layers; s->sp = *sp; s->sel = *sel;
    uniform(n_layers, *sel, s->mask);
    s->best_mask = s->mask;
    s->best_score = -1.0;
    s->active = true;
    s->rounds = 0; s->iters = 0; s->acc = 0;
    *out = s;
    return SSD_OK;
}

void ssd_search_destroy(ssd_search* s) { delete s; }

int ssd_search_mask(const ssd_search* s, uint8_t* mask_out)
{
    if (!s || !mask_out) return SSD_EINVAL;
    std::copy(s->mask.begin(), s->mask.end(), mask_out);
    return SSD_OK;
}

int ssd_search_status(const ssd_search* s, int32_t* rounds_out, double* best_score_out)
{
    if (!s) return SSD_EINVAL;
    if (rounds_out) *rounds_out = s->rounds;
    if (best_score_out) *best_score_out = s->best_score;
    return SSD_OK;
}

int ssd_search_observe(ssd_search* s, int n_accepted, const double* conf, uint8_t* mask_out, int32_t* active_out)
{
    if (!s || !mask_out || n_accepted < 0) return SSD_EINVAL;
    if (conf)
        for (int l = 0; l < s->L; l++)
            if (!std::isfinite(conf[l])) return SSD_EINVAL;
    auto finish = [&]() {
        std::copy(s->mask.begin(), s->mask.end(), mask_out);
        if (active_out) *active_out = s->active ? 1 : 0;
        return SSD_OK;
    };
    if (!s->active) return finish();
    if (conf) {
        s->ring.emplace_back(conf, conf + s->L);
        if ((int)s->ring.size() > s->sp.window) s->ring.pop_front();
    }
    s->acc += n_accepted;
    s->iters += 1;
    if (s->iters < s->sp.opt_interval) return finish();
    // the interval is over: score the current set by its mean accepted tokens per cycle
    const double score = (double)s->acc / (double)s->iters;
    s->iters = 0; s->acc = 0; s->rounds += 1;
    s->evaluated.insert(std::string(s->mask.begin(), s->mask.end()));
    if (score > s->best_score) { s->best_score = score; s->best_mask = s->mask; }
    if (score >= s->sp.score_goal || s->rounds >= s->sp.max_rounds || s->ring.empty()) {
        s->active = false;
        s->mask = s->best_mask;
        return finish();
    }
    std::vector<double> mean(s->L, 0.0);
    for (int l = 0; l < s->L; l++) {
        double t = 0.0;
        for (const auto& v : s->ring) t += v[l];
        mean[l] = t / (double)s->ring.size();
    }
    Selection S = select(mean.data(), s->L, s->sel);
    std::vector<uint8_t> cand_mask = S.mask;
    // a set that was already scored is shrunk: drop its member with the largest margin
    while (s->evaluated.count(std::string(cand_mask.begin(), cand_mask.end()))) {
        int members = 0, drop = -1;
        for (size_t i = 0; i < S.cand.size(); i++) {
            if (!cand_mask[S.cand[i]]) continue;
            members++;
            if (drop < 0 || S.margin[i] >= S.margin[drop]) drop = (int)i;  // ties: highest index
        }
        if (members <= S.n_min || drop < 0) {
            s->active = false;
            s->mask = s->best_mask;
            return finish();
        }
        cand_mask[S.cand[drop]] = 0;
    }
    s->mask = cand_mask;
    return finish();
}

}  // extern "C"
