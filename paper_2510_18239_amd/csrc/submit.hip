// Several independent requests handed to the GPU from several host threads at once.
//
// A request (lime_request) is four kernel launches, and a launch costs the host 2-3 us on this runtime: a serving loop
// that keeps a few requests in flight on as many streams spends 10-12 us of host time per request, which is most of
// the 17 us a request takes on the GPU and all of what the start of a burst waits for.  lime_request_many takes a list
// of requests and a list of streams, gives request i to stream i % n_streams, and submits the requests of each stream
// from a thread of its own: the caller's thread takes stream 0, a pool of library threads (created on first use, kept
// until the process ends) the others.  The launches of one stream stay in order; nothing else is shared.
#include "../../include/lime.h"

#include <string.h>

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "common.hpp"

namespace lime {
namespace {

constexpr int kMaxSubmitThreads = 8;

int32_t submit_one(const lime_request_args& r, void* stream) {
  return lime_request(r.E, r.lens, r.LC, r.lc_user_stride, r.Wq_hist, r.Wk_hist, r.Wv_hist, r.T, r.L, r.Wq_cand, r.Wk_cand,
                      r.Wv_cand, r.LP, r.O, r.B, r.N, r.C, r.d, r.h, r.m, r.scale_hist, r.scale_cand, r.xor_attention,
                      r.dtype, r.workspace, r.ws_bytes, stream);
}

// One batch at a time (callers are serialised); worker k submits the requests k, k + n_streams, ... of the batch.
class Submitter {
 public:
  static Submitter& instance() {
    static Submitter* s = new Submitter();  // never destroyed: its threads outlive every static destructor
    return *s;
  }

  int32_t run(const lime_request_args* reqs, int32_t n, void* const* streams, int32_t n_streams, char* message, size_t message_size) {
    std::lock_guard<std::mutex> one_batch(batch_mu_);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return LIME_LAUNCH_FAILED;
    const int helpers = std::min(std::min(n_streams, n) - 1, kMaxSubmitThreads - 1);
    {
      std::lock_guard<std::mutex> lock(mu_);
      while (static_cast<int>(workers_.size()) < helpers) {
        const int k = static_cast<int>(workers_.size()) + 1;
        workers_.emplace_back([this, k] { work(k); });
        workers_.back().detach();
      }
      reqs_ = reqs, n_ = n, streams_ = streams, n_streams_ = n_streams, device_ = device, helpers_ = helpers;
      status_ = LIME_OK, message_[0] = 0;
      pending_ = helpers;
      ++generation_;
    }
    wake_.notify_all();
    // the caller's share: stream 0, and the streams beyond the pool's size
    int32_t mine = LIME_OK;
    for (int s = 0; s < n_streams && mine == LIME_OK; s = s == 0 ? helpers + 1 : s + 1)
      for (int i = s; i < n && mine == LIME_OK; i += n_streams) mine = submit_one(reqs[i], streams[s]);
    if (mine != LIME_OK) record(mine, lime_last_error());
    std::unique_lock<std::mutex> lock(mu_);
    done_.wait(lock, [this] { return pending_ == 0; });
    if (status_ != LIME_OK && message != nullptr && message_size > 0) {
      strncpy(message, message_, message_size - 1);
      message[message_size - 1] = 0;
    }
    return status_;
  }

 private:
  void record(int32_t status, const char* text) {
    std::lock_guard<std::mutex> lock(mu_);
    if (status_ == LIME_OK) {
      status_ = status;
      strncpy(message_, text, sizeof(message_) - 1);
      message_[sizeof(message_) - 1] = 0;
    }
  }

  void work(int k) {
    uint64_t seen = 0;
    for (;;) {
      const lime_request_args* reqs;
      void* const* streams;
      int n, n_streams, device;
      {
        std::unique_lock<std::mutex> lock(mu_);
        wake_.wait(lock, [&] { return generation_ != seen; });
        seen = generation_;
        if (k > helpers_) continue;  // not part of this batch
        reqs = reqs_, streams = streams_, n = n_, n_streams = n_streams_, device = device_;
      }
      int32_t st = hipSetDevice(device) == hipSuccess ? LIME_OK : LIME_LAUNCH_FAILED;
      for (int i = k; i < n && st == LIME_OK; i += n_streams) st = submit_one(reqs[i], streams[k]);
      if (st != LIME_OK) record(st, st == LIME_LAUNCH_FAILED && lime_last_error()[0] == 0 ? "hipSetDevice failed" : lime_last_error());
      {
        std::lock_guard<std::mutex> lock(mu_);
        --pending_;
      }
      done_.notify_one();
    }
  }

  std::mutex batch_mu_, mu_;
  std::condition_variable wake_, done_;
  std::vector<std::thread> workers_;
  const lime_request_args* reqs_ = nullptr;
  void* const* streams_ = nullptr;
  int n_ = 0, n_streams_ = 0, device_ = 0, helpers_ = 0, pending_ = 0;
  uint64_t generation_ = 0;
  int32_t status_ = LIME_OK;
  char message_[512] = "";
};

}  // namespace
}  // namespace lime

extern "C" {
#pragma GCC visibility push(default)

int32_t lime_request_many(const lime_request_args* requests, int32_t n, void* const* streams, int32_t n_streams) {
  if (n < 0 || n_streams <= 0 || (n > 0 && (!requests || !streams)))
    return lime::set_error(LIME_INVALID_ARG, "lime_request_many: requests and streams must be given, n >= 0, n_streams > 0");
  if (n == 0) return LIME_OK;
  char message[512] = "";
  const int32_t st = lime::Submitter::instance().run(requests, n, streams, n_streams, message, sizeof(message));
  if (st != LIME_OK) return lime::set_error(st, message[0] ? message : "lime_request_many: a request failed");
  return LIME_OK;
}

#pragma GCC visibility pop
}
