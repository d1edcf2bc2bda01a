// Batch-firing policy of the inference scheduler (paper section 4.4): when to fire the pending
// pred calls as one GPU batch.  Host arithmetic only (IEEE doubles, one operation at a time, so
// that its decisions can be compared one by one with the CPU model's).
//
// The paper states the trade-off (too early: an under-used GPU; too late: waiting threads) and
// that the batch size follows the average call frequency through "models like Poisson process";
// the formulas are this build's:
//   rate    lambda = 1 / (exponentially weighted mean gap between arrivals)
//   service S(b) = a + c b microseconds, a least-squares line through exponentially weighted
//           moments of the (batch size, duration) pairs reported so far
//   target  b* = lambda a / (1 - lambda c): the batch size at which the expected arrivals during
//           one service period, lambda S(b), equal the batch; max_batch when lambda c >= 1
//   fire    when the GPU is idle: all pending calls (at most max_batch) if there are b* of them, if
//           the oldest has waited max_wait, or if (b* - pending) / lambda does not fit into what
//           is left of max_wait; otherwise wait.
#pragma once
#include <cstdint>
#include <deque>

namespace symkv {

class BatchTimer {
 public:
  BatchTimer(int32_t max_batch, double max_wait_us, double weight, double a_us, double c_us)
      : max_batch_(max_batch), max_wait_(max_wait_us), w_(weight), a_(a_us), c_(c_us) {}

  void arrive(double now_us);
  void done(int32_t n, double service_us);
  int32_t decide(double now_us, bool gpu_idle) const;
  void fired(int32_t n);
  double next_deadline() const;          // +inf when nothing is pending
  double rate() const;                   // calls per microsecond, 0 until two arrivals were seen
  double target() const;
  double a() const { return a_; }
  double c() const { return c_; }
  int64_t pending() const { return (int64_t)pending_.size(); }

 private:
  int32_t max_batch_;
  double max_wait_, w_, a_, c_;
  double mean_gap_ = 0.0, last_arrival_ = 0.0;
  int64_t n_gaps_ = 0, n_arrivals_ = 0, n_obs_ = 0;
  double mb_ = 0.0, ms_ = 0.0, mbb_ = 0.0, mbs_ = 0.0;
  std::deque<double> pending_;           // arrival times of the calls not yet fired
};

}  // namespace symkv
