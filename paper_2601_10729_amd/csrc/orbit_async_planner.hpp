// Background planner thread (Section 4: the Placement Planner runs in its own thread and solves
// one decode iteration ahead; the executor picks the finished plan up in the next iteration).
// One worker, one pending job (a newer submission replaces a job that has not started), one
// finished result (a newer result replaces one that was never collected).  Host only.
#pragma once

#include <condition_variable>
#include <cstdint>
#include <mutex>
#include <thread>
#include <vector>

#include "orbit_planner.hpp"

namespace orbit {

struct PlanJob {
  int64_t ticket = 0;
  int n_req = 0, L = 0, slots = 1;
  int64_t gpu_blocks = 0, max_evals = 0;
  double bandwidth = 0;
  bool stagger = false;
  std::vector<int64_t> blocks;
  std::vector<double> comp;
};

struct PlanDone {
  int64_t ticket = 0;
  int n_req = 0, L = 0;
  SearchResult res;
};

class AsyncPlanner {
 public:
  AsyncPlanner() : worker_([this] { run(); }) {}
  ~AsyncPlanner() {
    {
      std::lock_guard<std::mutex> g(mu_);
      stop_ = true;
    }
    cv_.notify_all();
    worker_.join();
  }

  int64_t submit(PlanJob job) {
    std::lock_guard<std::mutex> g(mu_);
    job.ticket = ++last_ticket_;
    pending_ = std::move(job);
    has_pending_ = true;
    cv_.notify_all();
    return last_ticket_;
  }

  // Takes the newest finished plan.  wait = true blocks until the newest submitted job is done
  // (returns false at once if nothing was ever submitted or everything was collected).
  bool poll(bool wait, PlanDone &out) {
    std::unique_lock<std::mutex> g(mu_);
    if (wait) cv_.wait(g, [&] { return (!has_pending_ && !busy_) || stop_; });
    if (!has_done_) return false;
    out = std::move(done_);
    has_done_ = false;
    return true;
  }

 private:
  void run() {
    for (;;) {
      PlanJob job;
      {
        std::unique_lock<std::mutex> g(mu_);
        cv_.wait(g, [&] { return has_pending_ || stop_; });
        if (stop_) return;
        job = std::move(pending_);
        has_pending_ = false;
        busy_ = true;
      }
      PlanDone d;
      d.ticket = job.ticket;
      d.n_req = job.n_req;
      d.L = job.L;
      d.res = plan_search(job.n_req, job.L, job.blocks.data(), job.gpu_blocks, job.slots, job.bandwidth,
                          job.comp.data(), job.max_evals, job.stagger);
      {
        std::lock_guard<std::mutex> g(mu_);
        done_ = std::move(d);
        has_done_ = true;
        busy_ = false;
      }
      cv_.notify_all();
    }
  }

  std::mutex mu_;
  std::condition_variable cv_;
  PlanJob pending_;
  PlanDone done_;
  bool has_pending_ = false, has_done_ = false, busy_ = false, stop_ = false;
  int64_t last_ticket_ = 0;
  std::thread worker_;  // declared last: starts after the state above exists
};

}  // namespace orbit
