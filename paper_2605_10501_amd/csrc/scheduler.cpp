// Wavefront sample scheduler (Sec. 3.4, Algorithm 1): host code, no device work.
//
// A sample is (t_f_bc, t_f_c, t_f_ac, t_b_bc, t_b_c, t_b_ac).  Three serial servers: PRE (sections in
// front of the critical one: forward t_f_bc, later backward t_b_ac), CRIT (t_f_c, t_b_c), POST (sections
// behind it: forward t_f_ac immediately followed by backward t_b_bc).  PRE's forward jobs have no
// predecessors and go first, so forward k of PRE finishes at the prefix sum of t_f_bc; everything else
// follows from "a job starts when its server is free and its predecessor on the sample's path is done",
// which for servers that keep schedule order is a chain of max / plus recurrences.
#include <algorithm>
#include <numeric>
#include <vector>

#include "common.h"

namespace {

struct Timeline {
    double makespan, critical_idle;
};

// order[k] indexes tuples; interleave != 0: the critical server runs forward and backward sample by
// sample, else all forwards in order, then all backwards in order.
Timeline simulate(const double *t, const int32_t *order, int n, int interleave) {
    Timeline r = {0.0, 0.0};
    if (n == 0) return r;
    double pre_fwd_all = 0.0;
    for (int k = 0; k < n; ++k) pre_fwd_all += t[6 * order[k] + 0];
    double pf = 0.0, c = 0.0, a = 0.0, p = pre_fwd_all, busy = 0.0;
    if (interleave) {
        for (int k = 0; k < n; ++k) {
            const double *s = t + 6 * order[k];
            pf += s[0];
            const double fe = std::max(c, pf) + s[1];                 // critical forward
            a = std::max(a, fe) + s[2] + s[3];                        // post-critical forward + backward
            c = a + s[4];                                             // critical backward (a >= fe)
            p = std::max(p, c) + s[5];                                // pre-critical backward
            busy += s[1] + s[4];
        }
    } else {
        std::vector<double> post_done(n);
        for (int k = 0; k < n; ++k) {
            const double *s = t + 6 * order[k];
            pf += s[0];
            c = std::max(c, pf) + s[1];
            a = std::max(a, c) + s[2] + s[3];
            post_done[k] = a;
            busy += s[1] + s[4];
        }
        for (int k = 0; k < n; ++k) {
            const double *s = t + 6 * order[k];
            c = std::max(c, post_done[k]) + s[4];
            p = std::max(p, c) + s[5];
        }
    }
    r.makespan = std::max(c, std::max(a, p));
    r.critical_idle = std::max(c - busy, 0.0);                        // the critical server ends at c and was busy `busy`
    return r;
}

// ---- O(1) evaluation of an insertion in the sample-by-sample mode --------------------------------------
// There one sample maps the state x = (front-forward sum, critical free, behind free, front free) to
//   pf' = pf + t0;  a' = max(a, max(c, pf') + t1) + t2 + t3;  c' = a' + t4;  p' = max(p, c') + t5,
// which is linear over the (max, +) semiring: x' = M (x) with a 4 x 4 matrix of sums of the sample's times.
// With the states after every prefix of the current order and the (max, +) products of every suffix, the
// makespan of "insert s at position pos" is  max over (c, a, p) of  Suffix[pos] (x) M_s (x) prefix[pos]:
// O(n) per sample to insert instead of O(n^2), O(n^2) for the whole schedule (the figure Sec. 3.4 quotes).
constexpr double NEG = -1e300;
struct Vec4 { double v[4]; };
struct Mat4 { double m[4][4]; };

Mat4 sample_matrix(const double *s) {
    Mat4 r;
    for (auto &row : r.m) for (double &e : row) e = NEG;
    const double t23 = s[2] + s[3];
    r.m[0][0] = s[0];                                                               // pf'
    r.m[2][0] = s[0] + s[1] + t23; r.m[2][1] = s[1] + t23; r.m[2][2] = t23;         // a'
    for (int j = 0; j < 3; ++j) r.m[1][j] = r.m[2][j] + s[4];                       // c' = a' + t4
    for (int j = 0; j < 3; ++j) r.m[3][j] = r.m[1][j] + s[5];                       // p' = max(p, c') + t5
    r.m[3][3] = s[5];
    return r;
}
Vec4 apply(const Mat4 &a, const Vec4 &x) {
    Vec4 r;
    for (int i = 0; i < 4; ++i) {
        double best = NEG;
        for (int j = 0; j < 4; ++j)
            if (a.m[i][j] > NEG / 2) best = std::max(best, a.m[i][j] + x.v[j]);
        r.v[i] = best;
    }
    return r;
}
Mat4 compose(const Mat4 &a, const Mat4 &b) {   // (a after b)
    Mat4 r;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            double best = NEG;
            for (int k = 0; k < 4; ++k)
                if (a.m[i][k] > NEG / 2 && b.m[k][j] > NEG / 2) best = std::max(best, a.m[i][k] + b.m[k][j]);
            r.m[i][j] = best;
        }
    return r;
}

// best insertion position of sample s into `result` (sample-by-sample mode); ties as in the plain search
int best_position_interleaved(const double *t, const std::vector<int32_t> &result, int32_t s) {
    const int m = (int)result.size();
    double front_sum = t[6 * s];
    for (int32_t k : result) front_sum += t[6 * k];
    std::vector<Vec4> prefix(m + 1);
    prefix[0] = Vec4{{0.0, 0.0, 0.0, front_sum}};                      // the front server's backward jobs start after all its forwards
    for (int k = 0; k < m; ++k) prefix[k + 1] = apply(sample_matrix(t + 6 * result[k]), prefix[k]);
    std::vector<Mat4> suffix(m + 1);
    for (auto &row : suffix[m].m) for (double &e : row) e = NEG;
    for (int i = 0; i < 4; ++i) suffix[m].m[i][i] = 0.0;               // identity
    for (int k = m - 1; k >= 0; --k) suffix[k] = compose(suffix[k + 1], sample_matrix(t + 6 * result[k]));
    const Mat4 ms = sample_matrix(t + 6 * s);
    int best_pos = 0;
    double best = 1e300;
    for (int pos = 0; pos <= m; ++pos) {
        const Vec4 x = apply(suffix[pos], apply(ms, prefix[pos]));
        const double mk = std::max(x.v[1], std::max(x.v[2], x.v[3]));
        if (mk < best * (1.0 - 1e-9)) { best = mk; best_pos = pos; }
    }
    return best_pos;
}

}  // namespace

extern "C" ms_status ms_schedule_makespan(int32_t n_samples, const double *tuples, const int32_t *order, int32_t interleave,
                                          double *makespan_out, double *critical_idle_out) {
    if (n_samples < 0 || (n_samples > 0 && (!tuples || !order))) return ms_fail(MS_ERR_INVALID_ARG, "schedule_makespan: bad argument");
    std::vector<char> seen(n_samples, 0);
    for (int k = 0; k < n_samples; ++k) {
        if (order[k] < 0 || order[k] >= n_samples || seen[order[k]])
            return ms_fail(MS_ERR_INVALID_ARG, "schedule_makespan: order is not a permutation of 0..%d", n_samples - 1);
        seen[order[k]] = 1;
    }
    for (long i = 0; i < 6L * n_samples; ++i)
        if (!(tuples[i] >= 0.0)) return ms_fail(MS_ERR_INVALID_ARG, "schedule_makespan: times must be non-negative numbers");
    const Timeline r = simulate(tuples, order, n_samples, interleave);
    if (makespan_out) *makespan_out = r.makespan;
    if (critical_idle_out) *critical_idle_out = r.critical_idle;
    return MS_OK;
}

extern "C" ms_status ms_schedule_samples(int32_t n_samples, const double *tuples, int32_t interleave, int32_t *order_out,
                                         double *makespan_out) {
    if (n_samples < 0 || (n_samples > 0 && (!tuples || !order_out))) return ms_fail(MS_ERR_INVALID_ARG, "schedule_samples: bad argument");
    for (long i = 0; i < 6L * n_samples; ++i)
        if (!(tuples[i] >= 0.0)) return ms_fail(MS_ERR_INVALID_ARG, "schedule_samples: times must be non-negative numbers");
    if (n_samples == 0) {
        if (makespan_out) *makespan_out = 0.0;
        return MS_OK;
    }
    // phase 1: ascending time before the critical section (stable: equal keys keep the input order)
    std::vector<int32_t> initial(n_samples);
    std::iota(initial.begin(), initial.end(), 0);
    std::stable_sort(initial.begin(), initial.end(), [&](int32_t x, int32_t y) { return tuples[6 * x] < tuples[6 * y]; });
    // phase 2: insert each remaining sample where the simulated makespan is least (first such position)
    std::vector<int32_t> result{initial[0]}, cand;
    for (int i = 1; i < n_samples; ++i) {
        const int32_t s = initial[i];
        const int m = (int)result.size();
        int best_pos = 0;
        if (interleave) {
            best_pos = best_position_interleaved(tuples, result, s);
        } else {
            double best = 1e300;
            cand.assign(m + 1, 0);
            for (int pos = 0; pos <= m; ++pos) {
                std::copy(result.begin(), result.begin() + pos, cand.begin());
                cand[pos] = s;
                std::copy(result.begin() + pos, result.end(), cand.begin() + pos + 1);
                const double mk = simulate(tuples, cand.data(), m + 1, interleave).makespan;
                if (mk < best * (1.0 - 1e-9)) { best = mk; best_pos = pos; }   // closer than 1e-9 relative: a tie
            }
        }
        result.insert(result.begin() + best_pos, s);
    }
    std::copy(result.begin(), result.end(), order_out);
    if (makespan_out) *makespan_out = simulate(tuples, result.data(), n_samples, interleave).makespan;
    return MS_OK;
}
