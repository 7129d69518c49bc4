// Node-local split controller (paper Sec. IV-A): once per decision epoch it observes the state vector of
// Table I and answers with a step of the EMB fraction out of the action set of Eq. 3; the next fraction is
// clip(alpha + step, 0.1, 0.9) (Eq. 4 / Eq. 6).  The paper's base policy is a PPO network trained offline on
// production traces and its Online Adapter a small residual network trained on line; neither the weights nor
// the traces are published, so the policy here is a stand-in that needs neither: a hill climb on the
// objective of Eq. 1, the measured P99 latency.  The Recovery Controller is the paper's rule as printed: a
// burst is an epoch whose latency exceeds the running mean of the last ten epochs by more than three
// standard deviations, and it is answered by moving memory towards the KV cache when the hot-user ratio is
// above 0.2.  Pure host C++, no device calls.
#pragma once

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>

namespace racer {

constexpr double kAlphaMin = 0.1, kAlphaMax = 0.9;          // Eq. 6
constexpr double kActionSteps[4] = {0.06, 0.04, 0.02, 0.0};  // magnitudes of the action set of Eq. 3
constexpr double kHotUserThreshold = 0.2;                    // rho* of the Recovery Controller
constexpr size_t kBurstWindow = 10;                          // epochs behind the latency baseline

struct AlphaState {  // Table I
  double hot_user_ratio, kv_hit_rate, emb_hit_rate, mean_seq_len, slo_violation, alpha, p99_latency_ms;
};

// Reward of one decision window (Eq. 5): SLO satisfaction less the tail penalty, lambda = 1 / tau_SLO.
inline double alpha_reward(double slo_satisfaction, double p99_latency_ms, double slo_ms) {
  const double over = p99_latency_ms - slo_ms;
  return slo_satisfaction - (over > 0.0 ? over / slo_ms : 0.0);
}

inline double clip_alpha(double a) { return a < kAlphaMin ? kAlphaMin : (a > kAlphaMax ? kAlphaMax : a); }

class AlphaController {
 public:
  explicit AlphaController(double slo_ms) : slo_ms_(slo_ms) {}

  // One epoch.  *step receives the action, the return value is the next fraction; *burst is set when the
  // Recovery Controller overrode the normal path.
  double decide(const AlphaState& s, double* step, int32_t* burst) {
    const double lat = s.p99_latency_ms;
    bool is_burst = false;
    if (window_.size() >= kBurstWindow / 2) {  // a baseline needs some history
      double mean = 0.0, var = 0.0;
      for (double v : window_) mean += v;
      mean /= static_cast<double>(window_.size());
      for (double v : window_) var += (v - mean) * (v - mean);
      // (the deviation is floored at 5 % of the baseline: on a quiet system the controller's own small probes
      // would otherwise count as bursts)
      const double sigma = std::max(std::sqrt(var / static_cast<double>(window_.size())), 0.05 * mean);
      is_burst = lat > mean + 3.0 * sigma;
    }
    window_.push_back(lat);
    if (window_.size() > kBurstWindow) window_.pop_front();
    double delta;
    if (is_burst) {
      // stability first: no probing during a burst; memory goes to the KV side if hot users dominate
      delta = s.hot_user_ratio > kHotUserThreshold ? -kActionSteps[0] : 0.0;
      level_ = 0;       // the climb starts over with the largest step once the burst has passed
      have_prev_ = false;
      hold_ = 0;
    } else {
      delta = climb(s);
    }
    double next = clip_alpha(s.alpha + delta);
    if (next == s.alpha && delta != 0.0) {  // the bound stopped the move: turn round
      dir_ = -dir_;
      delta = 0.0;
    }
    if (step) *step = delta;
    if (burst) *burst = is_burst ? 1 : 0;
    return next;
  }

  double slo_ms() const { return slo_ms_; }

 private:
  double climb(const AlphaState& s) {
    const double lat = s.p99_latency_ms;
    if (!have_prev_) {
      // first epoch (or the first after a burst): towards the cache that misses more
      dir_ = s.emb_hit_rate < s.kv_hit_rate ? 1.0 : -1.0;
      have_prev_ = true;
      prev_lat_ = lat;
      return dir_ * kActionSteps[level_];
    }
    const double tol = 0.02;  // changes below 2 % count as flat
    if (level_ == 3) {        // holding: probe again after a while, or at once if the latency drifts away
      const bool drift = lat > held_lat_ * (1.0 + 5.0 * tol);
      if (++hold_ >= 6 || drift) {
        level_ = 2;
        hold_ = 0;
        prev_lat_ = lat;
        return dir_ * kActionSteps[level_];
      }
      return 0.0;
    }
    if (lat < prev_lat_ * (1.0 - tol)) {
      // the last step helped: same direction, same size
    } else if (lat > prev_lat_ * (1.0 + tol)) {
      dir_ = -dir_;  // it hurt: back, with the next smaller step
      level_ += 1;
    } else {
      level_ += 1;   // flat: a smaller step the same way
    }
    prev_lat_ = lat;
    if (level_ >= 3) {
      level_ = 3;
      held_lat_ = lat;
      hold_ = 0;
      return 0.0;
    }
    return dir_ * kActionSteps[level_];
  }

  double slo_ms_;
  std::deque<double> window_;
  bool have_prev_ = false;
  double prev_lat_ = 0.0, held_lat_ = 0.0, dir_ = -1.0;
  int level_ = 0;  // index into kActionSteps
  int hold_ = 0;
};

}  // namespace racer
