// Batch-firing policy of the inference scheduler (paper section 4.4).  See sched.hpp.
#include "sched.hpp"

#include <algorithm>
#include <limits>

// every product and sum is rounded on its own, as in the CPU model
#pragma clang fp contract(off)

namespace symkv {

void BatchTimer::arrive(double now_us) {
  if (n_arrivals_ > 0) {
    const double gap = now_us - last_arrival_;
    if (n_gaps_ == 0) mean_gap_ = gap;
    else mean_gap_ = mean_gap_ + w_ * (gap - mean_gap_);
    ++n_gaps_;
  }
  ++n_arrivals_;
  last_arrival_ = now_us;
  pending_.push_back(now_us);
}

void BatchTimer::done(int32_t n, double service_us) {
  const double b = (double)n, s = service_us;
  if (n_obs_ == 0) {
    mb_ = b;
    ms_ = s;
    mbb_ = b * b;
    mbs_ = b * s;
  } else {
    mb_ = mb_ + w_ * (b - mb_);
    ms_ = ms_ + w_ * (s - ms_);
    mbb_ = mbb_ + w_ * (b * b - mbb_);
    mbs_ = mbs_ + w_ * (b * s - mbs_);
  }
  ++n_obs_;
  const double var = mbb_ - mb_ * mb_;
  if (var > 1e-9 * mbb_) {                      // batch sizes differ enough for a slope
    const double c = (mbs_ - mb_ * ms_) / var;
    c_ = c > 0.0 ? c : 0.0;
  }
  const double a = ms_ - c_ * mb_;
  a_ = a > 0.0 ? a : 0.0;
}

double BatchTimer::rate() const { return (n_gaps_ > 0 && mean_gap_ > 0.0) ? 1.0 / mean_gap_ : 0.0; }

double BatchTimer::target() const {
  const double lam = rate();
  const double load = lam * c_;
  if (load >= 1.0) return (double)max_batch_;
  const double t = lam * a_ / (1.0 - load);
  return std::min(std::max(t, 1.0), (double)max_batch_);
}

int32_t BatchTimer::decide(double now_us, bool gpu_idle) const {
  if (!gpu_idle || pending_.empty()) return 0;
  const int32_t q = (int32_t)std::min<int64_t>((int64_t)pending_.size(), max_batch_);
  const double lam = rate();
  if (lam <= 0.0) return q;                     // no rate known yet: nothing to wait for
  const double waited = now_us - pending_.front();
  const double left = max_wait_ - waited;
  if (left <= 0.0) return q;
  const double missing = target() - (double)q;
  if (missing <= 0.0) return q;
  if (missing / lam > left) return q;           // the target is out of reach before the deadline
  return 0;
}

void BatchTimer::fired(int32_t n) {
  for (int32_t i = 0; i < n && !pending_.empty(); ++i) pending_.pop_front();
}

double BatchTimer::next_deadline() const {
  return pending_.empty() ? std::numeric_limits<double>::infinity() : pending_.front() + max_wait_;
}

}  // namespace symkv
