// SushiSched (paper Algorithm 1, Section 3.3), host side.
//
// Per query: under STRICT_ACCURACY serve the lowest-latency SubNet among those accurate enough,
// under STRICT_LATENCY the most accurate among those fast enough, where "latency" is the table
// entry for (SubNet, currently cached SubGraph).  Across queries: keep the element-wise sum of the
// last Q served vectors and, after every Q-th query, pick the candidate nearest to their mean.
// The distance is compared exactly: with n vectors in the window, sum_k (n*g[k] - sum[k])^2 in
// 64-bit integers is n^2 times the squared Euclidean distance to the mean.  Ties go to the lowest
// index.  If no SubNet meets the hard constraint, the most accurate (STRICT_ACCURACY) or the
// fastest (STRICT_LATENCY) one is served.
#include "sched.h"

namespace sushi {

int Scheduler::init(const sushi_sched_desc &d, std::string &err) {
    ready_ = false;
    if (d.n_subnets < 1 || d.n_subgraphs < 0 || d.vec_len < 1 || d.Q < 1 || !d.subnet_vecs || !d.accuracy ||
        !d.table || (d.n_subgraphs > 0 && !d.subgraph_vecs)) {
        err = "sched: bad descriptor";
        return SUSHI_EINVAL;
    }
    if (d.policy != SUSHI_STRICT_ACCURACY && d.policy != SUSHI_STRICT_LATENCY) {
        err = "sched: unknown policy";
        return SUSHI_EINVAL;
    }
    if (d.initial_cache < -1 || d.initial_cache >= d.n_subgraphs) {
        err = "sched: initial cache index out of range";
        return SUSHI_EINVAL;
    }
    n_ = d.n_subnets, m_ = d.n_subgraphs, len_ = d.vec_len, q_ = d.Q, policy_ = d.policy, cache_ = d.initial_cache;
    v_.assign(d.subnet_vecs, d.subnet_vecs + (size_t)n_ * len_);
    g_.assign(d.subgraph_vecs, d.subgraph_vecs + (size_t)m_ * len_);
    acc_.assign(d.accuracy, d.accuracy + n_);
    table_.assign(d.table, d.table + (size_t)n_ * (m_ + 1));
    window_.clear();
    sums_.assign(len_, 0);
    t_ = 0;
    ready_ = true;
    return SUSHI_OK;
}

int Scheduler::select(float a_t, float l_t) const {
    const int col = cache_ < 0 ? m_ : cache_;
    auto lat = [&](int i) { return table_[(size_t)i * (m_ + 1) + col]; };
    int best = -1;
    if (policy_ == SUSHI_STRICT_ACCURACY) {
        for (int i = 0; i < n_; ++i)
            if (acc_[i] >= a_t && (best < 0 || lat(i) < lat(best))) best = i;
        if (best < 0)
            for (int i = 0; i < n_; ++i)
                if (best < 0 || acc_[i] > acc_[best]) best = i;
    } else {
        for (int i = 0; i < n_; ++i)
            if (lat(i) <= l_t && (best < 0 || acc_[i] > acc_[best])) best = i;
        if (best < 0)
            for (int i = 0; i < n_; ++i)
                if (best < 0 || lat(i) < lat(best)) best = i;
    }
    return best;
}

int Scheduler::record(const int32_t *vec) {
    window_.emplace_back(vec, vec + len_);
    for (int k = 0; k < len_; ++k) sums_[k] += vec[k];
    if ((int)window_.size() > q_) {
        const std::vector<int32_t> &old = window_.front();
        for (int k = 0; k < len_; ++k) sums_[k] -= old[k];
        window_.pop_front();
    }
    ++t_;
    if (t_ % (uint64_t)q_ != 0 || m_ == 0) return -1;
    const int64_t n = (int64_t)window_.size();
    int best = -1;
    int64_t best_d = 0;
    for (int j = 0; j < m_; ++j) {
        const int32_t *g = &g_[(size_t)j * len_];
        int64_t d = 0;
        for (int k = 0; k < len_; ++k) {
            const int64_t e = n * g[k] - sums_[k];
            d += e * e;
        }
        if (best < 0 || d < best_d) best = j, best_d = d;
    }
    cache_ = best;
    return best;
}

}  // namespace sushi
