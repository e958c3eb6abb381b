// Checkpoint placement layer (host code): Table 1 placements, Sec. 3 metrics, the O(N M)
// dynamic program of Theorem 2, the exponentially weighted overlap histogram of Sec. 4.2.
#include "ckpt_place.h"

#include <cmath>
#include <cstring>
#include <limits>
#include <vector>

#include "gdn_resume.h"

namespace {

bool increasing_in_range(const int32_t* pos, int32_t n, int32_t N) {
    for (int32_t i = 0; i < n; ++i) {
        if (pos[i] < 1 || pos[i] > N) return false;
        if (i > 0 && pos[i] <= pos[i - 1]) return false;
    }
    return true;
}

int32_t isqrt32(int32_t n) {
    int32_t s = (int32_t)std::sqrt((double)n);
    while ((int64_t)s * s > n) --s;
    while ((int64_t)(s + 1) * (s + 1) <= n) ++s;
    return s;
}

// One layer of Theorem 2's recurrence.  With P_j = sum_{t<=j} p_t and T_j = sum_{t<=j} t p_t,
//   dp[m, j] = T_j + min_{1<=s<=j} ( b_s - s P_j ),   b_s = dp[m-1, s-1] - T_{s-1} + s P_{s-1}:
// candidate s is the line y = -s x + b_s queried at x = P_j.  Slopes decrease with s and the
// queries do not decrease with j, so the lower envelope is kept in a deque whose front only
// moves forward.  Line s becomes available at j = s.
struct Line { double b; int32_t s; };

inline double value(const Line& l, double x) { return l.b - (double)l.s * x; }

// true when `mid` is nowhere strictly below both neighbours (slopes: lo > mid > hi)
inline bool redundant(const Line& lo, const Line& mid, const Line& hi) {
    // intersection(lo, hi) at x = (hi.b - lo.b) / (hi.s - lo.s); mid is useless if its value there is not smaller
    const double lhs = (hi.b - lo.b) * (double)(mid.s - lo.s);
    const double rhs = (mid.b - lo.b) * (double)(hi.s - lo.s);
    return lhs <= rhs;
}

void dp_layer(const std::vector<double>& prev, const std::vector<double>& P, const std::vector<double>& T, int32_t N,
              std::vector<double>& cur, int32_t* arg) {
    std::vector<Line> hull;
    hull.reserve((size_t)N);
    size_t front = 0;
    cur[0] = 0.0;
    for (int32_t j = 1; j <= N; ++j) {
        const Line nl{prev[j - 1] - T[j - 1] + (double)j * P[j - 1], j};
        while (hull.size() - front >= 2 && redundant(hull[hull.size() - 2], hull.back(), nl)) hull.pop_back();
        hull.push_back(nl);
        if (front >= hull.size()) front = hull.size() - 1;
        const double x = P[j];
        while (front + 1 < hull.size() && value(hull[front + 1], x) <= value(hull[front], x)) ++front;
        cur[j] = T[j] + value(hull[front], x);
        arg[j] = hull[front].s;
    }
}

}  // namespace

struct ckpt_hist {
    int32_t N;
    double gamma;
    double scale;            // true weight = scale * w
    double norm;             // sum of true weights
    int64_t n;
    std::vector<double> w;
};

extern "C" {

int32_t ckpt_place_balanced(int32_t N, int32_t M, int32_t* pos) {
    if (N < 1 || M < 0 || M > N) return GDN_ERR_COUNT;
    if (M > 0 && !pos) return GDN_ERR_NULL;
    for (int32_t i = 1; i <= M; ++i) pos[i - 1] = (int32_t)(((int64_t)i * (N + 1)) / (M + 1));
    return M;
}

int32_t ckpt_place_block(int32_t N, int32_t B, int32_t* pos, int32_t capacity) {
    if (N < 1 || B < 1) return GDN_ERR_COUNT;
    const int32_t n = N / B;
    if (n > capacity) return GDN_ERR_WORKSPACE;
    if (n > 0 && !pos) return GDN_ERR_NULL;
    for (int32_t i = 1; i <= n; ++i) pos[i - 1] = i * B;
    return n;
}

int32_t ckpt_place_sqrt(int32_t N, int32_t* pos, int32_t capacity) {
    if (N < 1) return GDN_ERR_COUNT;
    return ckpt_place_block(N, isqrt32(N), pos, capacity);
}

int32_t ckpt_place_log(int32_t N, int32_t unit, int32_t M, int32_t* pos) {
    if (N < 1 || unit < 1 || M < 0) return GDN_ERR_COUNT;
    if (M > 0 && !pos) return GDN_ERR_NULL;
    int32_t n = 0;
    int64_t span = 2;                                   // 2^i
    while (n < M && (int64_t)unit * (span - 1) <= N) {
        pos[n++] = (int32_t)((int64_t)unit * (span - 1));
        span *= 2;
    }
    return n;
}

int32_t ckpt_clip_to_blocks(const int32_t* pos, int32_t n, int32_t B, int32_t* out) {
    if (n < 0 || B < 1) return GDN_ERR_COUNT;
    if (n > 0 && (!pos || !out)) return GDN_ERR_NULL;
    if (!increasing_in_range(pos, n, std::numeric_limits<int32_t>::max())) return GDN_ERR_EMIT;
    int32_t m = 0;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t c = pos[i] / B * B;
        if (c > 0 && (m == 0 || out[m - 1] != c)) out[m++] = c;
    }
    return m;
}

int32_t ckpt_expected_recompute(const double* p, int32_t N, const int32_t* pos, int32_t n, double* expected,
                                double* no_cache, double* savings, double* reduction) {
    if (N < 1 || n < 0) return GDN_ERR_COUNT;
    if (!p || (n > 0 && !pos)) return GDN_ERR_NULL;
    if (!increasing_in_range(pos, n, N)) return GDN_ERR_EMIT;
    double e = 0.0, r = 0.0;
    int32_t k = 0, l = 0;                               // l = deepest checkpoint <= t
    for (int32_t t = 1; t <= N; ++t) {
        if (p[t - 1] < 0.0 || p[t - 1] != p[t - 1]) return GDN_ERR_COUNT;
        while (k < n && pos[k] <= t) l = pos[k++];
        e += p[t - 1] * (double)(t - l);
        r += p[t - 1] * (double)t;
    }
    if (expected) *expected = e;
    if (no_cache) *no_cache = r;
    if (savings) *savings = r > 0.0 ? 1.0 - e / r : 0.0;
    if (reduction) *reduction = e > 0.0 ? r / e : std::numeric_limits<double>::infinity();
    return GDN_OK;
}

int32_t ckpt_place_dp(const double* p, int32_t N, int32_t M, int32_t* pos, double* cost) {
    if (N < 1 || M < 0) return GDN_ERR_COUNT;
    if (!p || (M > 0 && !pos)) return GDN_ERR_NULL;
    if (M > N) M = N;
    if ((int64_t)M * (N + 1) > ((int64_t)1 << 31)) return GDN_ERR_COUNT;   // back-pointer table size
    std::vector<double> P((size_t)N + 1, 0.0), T((size_t)N + 1, 0.0);
    for (int32_t t = 1; t <= N; ++t) {
        if (p[t - 1] < 0.0 || p[t - 1] != p[t - 1]) return GDN_ERR_COUNT;
        P[t] = P[t - 1] + p[t - 1];
        T[t] = T[t - 1] + p[t - 1] * (double)t;
    }
    std::vector<double> prev(T), cur((size_t)N + 1, 0.0);                   // dp[0, j] = T_j
    std::vector<int32_t> arg((size_t)M * ((size_t)N + 1), 0);
    for (int32_t m = 1; m <= M; ++m) {
        dp_layer(prev, P, T, N, cur, arg.data() + (size_t)(m - 1) * ((size_t)N + 1));
        prev.swap(cur);
    }
    if (cost) *cost = prev[N];
    // walk the back-pointers: the last checkpoint serving depths 1..j with m checkpoints
    std::vector<int32_t> rev;
    int32_t j = N;
    for (int32_t m = M; m >= 1 && j >= 1; --m) {
        const int32_t s = arg[(size_t)(m - 1) * ((size_t)N + 1) + j];
        rev.push_back(s);
        j = s - 1;
    }
    const int32_t n = (int32_t)rev.size();
    for (int32_t i = 0; i < n; ++i) pos[i] = rev[n - 1 - i];
    return n;
}

ckpt_hist* ckpt_hist_create(int32_t N, double gamma) {
    if (N < 1 || !(gamma > 0.0) || gamma > 1.0) return nullptr;
    ckpt_hist* h = new (std::nothrow) ckpt_hist;
    if (!h) return nullptr;
    h->N = N; h->gamma = gamma; h->scale = 1.0; h->norm = 0.0; h->n = 0;
    h->w.assign((size_t)N, 0.0);
    return h;
}

void ckpt_hist_destroy(ckpt_hist* h) { delete h; }

int64_t ckpt_hist_observe(ckpt_hist* h, int32_t t) {
    if (!h) return GDN_ERR_NULL;
    if (t < 1 || t > h->N) return GDN_ERR_COUNT;
    // every earlier weight is multiplied by gamma: done lazily through the common scale
    h->scale *= h->gamma;
    h->norm = h->norm * h->gamma + 1.0;
    if (h->scale < 1e-200) {                             // fold the scale back in before it underflows
        for (double& x : h->w) x *= h->scale;
        h->scale = 1.0;
    }
    h->w[(size_t)t - 1] += 1.0 / h->scale;
    return ++h->n;
}

int32_t ckpt_hist_get(const ckpt_hist* h, double* p) {
    if (!h || !p) return GDN_ERR_NULL;
    const double f = h->norm > 0.0 ? h->scale / h->norm : 0.0;
    for (int32_t t = 0; t < h->N; ++t) p[t] = h->w[(size_t)t] * f;
    return GDN_OK;
}

int32_t ckpt_hist_solve(const ckpt_hist* h, int32_t M, int32_t B, int32_t* pos, double* cost) {
    if (!h) return GDN_ERR_NULL;
    if (B < 1) return GDN_ERR_COUNT;
    std::vector<double> p((size_t)h->N);
    int32_t rc = ckpt_hist_get(h, p.data());
    if (rc != GDN_OK) return rc;
    std::vector<int32_t> raw((size_t)(M > 0 ? M : 1));
    const int32_t n = ckpt_place_dp(p.data(), h->N, M, M > 0 ? raw.data() : nullptr, cost);
    if (n < 0) return n;
    if (M > 0 && !pos) return GDN_ERR_NULL;
    if (B == 1) {
        std::memcpy(pos, raw.data(), sizeof(int32_t) * (size_t)n);
        return n;
    }
    return ckpt_clip_to_blocks(raw.data(), n, B, pos);
}

// ---- the online loop of Sec. 5 ("Our method"): observe, re-solve every `period` requests
struct ckpt_online {
    ckpt_hist* hist;
    int32_t M, B, period;
    std::vector<int32_t> pos;
    int64_t solves;
};

ckpt_online* ckpt_online_create(int32_t N, int32_t M, int32_t B, double gamma, int32_t period) {
    if (M < 1 || B < 1 || period < 1) return nullptr;
    ckpt_hist* h = ckpt_hist_create(N, gamma);
    if (!h) return nullptr;
    ckpt_online* o = new (std::nothrow) ckpt_online;
    if (!o) {
        ckpt_hist_destroy(h);
        return nullptr;
    }
    o->hist = h; o->M = M; o->B = B; o->period = period; o->solves = 0;
    return o;
}

void ckpt_online_destroy(ckpt_online* o) {
    if (!o) return;
    ckpt_hist_destroy(o->hist);
    delete o;
}

int32_t ckpt_online_observe(ckpt_online* o, int32_t t) {
    if (!o) return GDN_ERR_NULL;
    const int64_t n = ckpt_hist_observe(o->hist, t);
    if (n < 0) return (int32_t)n;
    if (n % o->period != 0) return 0;
    std::vector<int32_t> next((size_t)o->M);
    const int32_t k = ckpt_hist_solve(o->hist, o->M, o->B, next.data(), nullptr);
    if (k < 0) return k;
    next.resize((size_t)k);
    o->pos.swap(next);
    o->solves += 1;
    return 1;
}

int32_t ckpt_online_schedule(const ckpt_online* o, int32_t* pos, int32_t capacity) {
    if (!o) return GDN_ERR_NULL;
    const int32_t n = (int32_t)o->pos.size();
    if (n > capacity) return GDN_ERR_WORKSPACE;
    if (n > 0 && !pos) return GDN_ERR_NULL;
    if (n > 0) std::memcpy(pos, o->pos.data(), sizeof(int32_t) * (size_t)n);
    return n;
}

const ckpt_hist* ckpt_online_histogram(const ckpt_online* o) { return o ? o->hist : nullptr; }

}  // extern "C"
