// Host-side SushiSched: per-query SubNet selection and every-Q SubGraph choice
// (paper Algorithm 1 and Section 3.3).
#pragma once

#include <cstdint>
#include <deque>
#include <string>
#include <vector>

#include "../../include/sushi.h"

namespace sushi {

class Scheduler {
  public:
    int init(const sushi_sched_desc &d, std::string &err);
    bool ready() const { return ready_; }
    int vec_len() const { return len_; }
    // SubNet for a query (A_t, L_t) under the current cache state.
    int select(float acc_target, float lat_target) const;
    // Accounts one served vector; returns the candidate chosen on a Q-th query, else -1.
    int record(const int32_t *vec);
    const int32_t *subnet_vec(int i) const { return &v_[(size_t)i * len_]; }

  private:
    bool ready_ = false;
    int n_ = 0, m_ = 0, len_ = 0, q_ = 1, policy_ = SUSHI_STRICT_LATENCY, cache_ = -1;
    uint64_t t_ = 0;
    std::vector<int32_t> v_, g_;
    std::vector<float> acc_, table_;
    std::deque<std::vector<int32_t>> window_;
    std::vector<int64_t> sums_;
};

}  // namespace sushi
