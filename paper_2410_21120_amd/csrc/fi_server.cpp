// Request aggregation in front of a loaded DAG (Section IV, "Manager": requests for the member models
// arrive one by one; those that arrive while the device is busy are gathered, per model, into the batch of the
// next pass).  Every lane of the DAG (the members of one architecture) has a worker thread with a stream of
// its own: it takes up to max_batch waiting requests of each of its members, copies their images into the
// members' batch buffers, runs ONE fi_run_lane pass, copies every output row to its request's buffer and wakes
// the waiters.  While that pass is in flight new requests queue up: the busier the device, the larger the
// batches.  Lanes share no tensor, so their passes overlap freely on the device and a short model never waits
// for a long one; members of one lane travel in the same grouped launches.  Host logic only: every device
// step is a copy kernel or the public fi_run_lane / fi_swap_model.
#include <hip/hip_runtime.h>

#include <chrono>
#include <condition_variable>
#include <deque>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <unordered_set>
#include <vector>

#include "fi_internal.h"

using namespace fi;

namespace {

double now_ms() {
  using clk = std::chrono::steady_clock;
  return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

struct Request {
  uint64_t ticket;
  const void* d_image;
  void* d_output;
  double t_submit;
};

struct LaneWorker {
  int32_t lane = 0;
  std::vector<int32_t> members;   // the lane's members
  hipStream_t stream = nullptr;
  std::thread thread;
  std::condition_variable cv;     // signalled when one of the lane's members gets a request
};

}  // namespace

struct fi_server {
  fi_dag* dag = nullptr;
  ServingInfo info;
  fi_server_opts opts{};
  int device = 0;
  std::vector<uint8_t*> in_buf, out_buf;    // per member: max_batch images / max_batch output rows (device)
  std::vector<std::unique_ptr<LaneWorker>> workers;
  std::mutex mu;
  std::condition_variable cv_done;          // a pass finished, a swap finished
  std::vector<std::deque<Request>> queue;   // per member, first in first out
  std::vector<int32_t> in_flight;           // per member: requests taken by a pass that has not finished
  std::unordered_set<uint64_t> pending;     // tickets submitted and not yet served
  uint64_t next_ticket = 1;
  bool stopping = false;                    // serve what is queued, then leave
  bool regroup = false;                     // a member swap needs every worker to leave after its current pass
  bool swapping = false;
  int32_t swap_slot = -1;
  fi_status failed = FI_OK;                 // first error of a worker; every later wait reports it
  std::string failure;
  // statistics (under mu)
  uint64_t n_requests = 0, n_passes = 0, max_images = 0;
  double sum_latency_ms = 0.0, max_latency_ms = 0.0, busy_ms = 0.0;

  void* dev_alloc(size_t n) const {
    if (info.opts.dev_alloc) return info.opts.dev_alloc(n, info.opts.user);
    void* p = nullptr;
    if (hipMalloc(&p, n) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return p;
  }
  void dev_free(void* p) const {
    if (!p) return;
    if (info.opts.dev_free) info.opts.dev_free(p, info.opts.user); else (void)hipFree(p);
  }
  void fail(fi_status st, const std::string& why) {   // under mu
    if (failed == FI_OK) { failed = st; failure = why; }
  }
  size_t waiting_in(const LaneWorker& w) const {      // under mu
    size_t k = 0;
    for (int32_t m : w.members) k += queue[(size_t)m].size();
    return k;
  }
  fi_status start_workers();
  void join_workers();
  void release() {
    for (uint8_t* p : in_buf) dev_free(p);
    for (uint8_t* p : out_buf) dev_free(p);
    in_buf.clear(); out_buf.clear();
  }
  void serve(LaneWorker* w);
};

void fi_server::serve(LaneWorker* w) {
  (void)hipSetDevice(device);
  const int32_t n = info.n_models;
  std::vector<std::vector<Request>> take((size_t)n);
  std::vector<const void*> ins((size_t)n, nullptr);
  std::vector<void*> outs((size_t)n, nullptr);
  std::vector<int32_t> batches((size_t)n, 0);
  std::vector<const void*> csrc;
  std::vector<void*> cdst;
  const size_t lane_cap = w->members.size() * (size_t)info.max_batch;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(mu);
      w->cv.wait(lk, [&] { return waiting_in(*w) > 0 || stopping || regroup; });
      // When the workers are called off for a swap, nothing new is started: the queue of the outgoing
      // member has been served before that, every other request waits for the new workers.
      if (regroup) return;
      if (waiting_in(*w) == 0) { if (stopping) return; continue; }
      if (opts.max_wait_us > 0 && !stopping) {
        // a first request after an idle period: give its companions a moment to arrive
        const auto until = std::chrono::system_clock::now() + std::chrono::microseconds(opts.max_wait_us);
        w->cv.wait_until(lk, until, [&] { return stopping || regroup || waiting_in(*w) >= lane_cap; });
        if (regroup) return;
      }
      for (int32_t m : w->members) {
        take[(size_t)m].clear();
        std::deque<Request>& q = queue[(size_t)m];
        while (!q.empty() && (int32_t)take[(size_t)m].size() < info.max_batch) { take[(size_t)m].push_back(q.front()); q.pop_front(); }
        in_flight[(size_t)m] += (int32_t)take[(size_t)m].size();
      }
    }
    const double t0 = now_ms();
    hipError_t e = hipSuccess;
    uint64_t images = 0;
    // gather: the images of every member's requests into that member's batch buffer.  Rows that allow it (16-byte
    // aligned, a multiple of 16 bytes long) travel in one copy kernel per kCopyRows rows, the others one by one.
    csrc.clear(); cdst.clear();
    for (int32_t m : w->members) {
      batches[(size_t)m] = (int32_t)take[(size_t)m].size();
      ins[(size_t)m] = in_buf[(size_t)m];
      outs[(size_t)m] = out_buf[(size_t)m];
      images += take[(size_t)m].size();
      for (size_t i = 0; i < take[(size_t)m].size() && e == hipSuccess; ++i) {
        uint8_t* to = in_buf[(size_t)m] + i * info.image_bytes;
        const void* from = take[(size_t)m][i].d_image;
        if (info.image_bytes % 16 == 0 && ((reinterpret_cast<uintptr_t>(from) | reinterpret_cast<uintptr_t>(to)) & 15) == 0) { csrc.push_back(from); cdst.push_back(to); }
        else e = hipMemcpyAsync(to, from, (size_t)info.image_bytes, hipMemcpyDeviceToDevice, w->stream);
      }
    }
    if (e == hipSuccess && !csrc.empty()) e = (hipError_t)launch_copy_rows(csrc.data(), cdst.data(), (int32_t)csrc.size(), info.image_bytes, w->stream);
    fi_status st = e == hipSuccess ? fi_run_lane(dag, w->lane, ins.data(), batches.data(), outs.data(), w->stream) : FI_EHIP;
    std::string why = st != FI_OK ? (e != hipSuccess ? std::string("gathering the images: ") + hipGetErrorString(e) : std::string(fi_last_error())) : std::string();
    // scatter: every output row to its request's buffer (rows of one length share a copy kernel)
    for (size_t k = 0; k < w->members.size() && st == FI_OK; ++k) {
      const int32_t m = w->members[k];
      csrc.clear(); cdst.clear();
      const uint64_t ob = info.out_bytes[(size_t)m];
      for (size_t i = 0; i < take[(size_t)m].size() && st == FI_OK; ++i) {
        const uint8_t* from = out_buf[(size_t)m] + i * ob;
        void* to = take[(size_t)m][i].d_output;
        if (ob % 16 == 0 && ((reinterpret_cast<uintptr_t>(from) | reinterpret_cast<uintptr_t>(to)) & 15) == 0) { csrc.push_back(from); cdst.push_back(to); continue; }
        e = hipMemcpyAsync(to, from, (size_t)ob, hipMemcpyDeviceToDevice, w->stream);
        if (e != hipSuccess) { st = FI_EHIP; why = std::string("hipMemcpyAsync: ") + hipGetErrorString(e); }
      }
      if (st == FI_OK && !csrc.empty()) {
        e = (hipError_t)launch_copy_rows(csrc.data(), cdst.data(), (int32_t)csrc.size(), ob, w->stream);
        if (e != hipSuccess) { st = FI_EHIP; why = std::string("scattering the outputs: ") + hipGetErrorString(e); }
      }
    }
    e = hipStreamSynchronize(w->stream);
    if (e != hipSuccess && st == FI_OK) { st = FI_EHIP; why = std::string("hipStreamSynchronize: ") + hipGetErrorString(e); }
    const double t1 = now_ms();
    {
      std::lock_guard<std::mutex> lk(mu);
      if (st != FI_OK) fail(st, why);
      for (int32_t m : w->members) {
        for (const Request& r : take[(size_t)m]) {
          pending.erase(r.ticket);
          const double lat = t1 - r.t_submit;
          sum_latency_ms += lat;
          if (lat > max_latency_ms) max_latency_ms = lat;
          ++n_requests;
        }
        in_flight[(size_t)m] -= (int32_t)take[(size_t)m].size();
        take[(size_t)m].clear();
      }
      ++n_passes;
      if (images > max_images) max_images = images;
      busy_ms += t1 - t0;
    }
    cv_done.notify_all();
  }
}

// One worker per lane of the DAG as it is now (a member swap may have changed the lanes).
fi_status fi_server::start_workers() {
  workers.clear();
  for (int32_t l = 0; l < info.n_lanes; ++l) {
    std::unique_ptr<LaneWorker> w(new LaneWorker);
    w->lane = l;
    for (int32_t m = 0; m < info.n_models; ++m)
      if (info.lane[(size_t)m] == l) w->members.push_back(m);
    if (w->members.empty()) continue;
    if (hipStreamCreateWithFlags(&w->stream, hipStreamNonBlocking) != hipSuccess) {
      (void)hipGetLastError();
      for (auto& made : workers) (void)hipStreamDestroy(made->stream);
      workers.clear();
      return FI_EHIP;
    }
    workers.push_back(std::move(w));
  }
  for (auto& w : workers) {
    LaneWorker* p = w.get();
    p->thread = std::thread([this, p] { serve(p); });
  }
  return FI_OK;
}

// The caller has set `stopping` or `regroup` (under mu, released since): every worker leaves after its current pass.
void fi_server::join_workers() {
  std::vector<std::unique_ptr<LaneWorker>> leaving;
  {
    std::lock_guard<std::mutex> lk(mu);   // fi_server_submit walks the list under the same lock
    leaving.swap(workers);
  }
  for (auto& w : leaving) w->cv.notify_all();
  for (auto& w : leaving) {
    if (w->thread.joinable()) w->thread.join();
    if (w->stream) { (void)hipStreamDestroy(w->stream); w->stream = nullptr; }
  }
}

extern "C" {

fi_status fi_server_start(fi_dag* dag, const fi_server_opts* opts, fi_server** out) {
  if (!dag || !out) { set_error("null argument"); return FI_EINVAL; }
  if (opts && opts->max_wait_us < 0) { set_error("max_wait_us must be >= 0"); return FI_EINVAL; }
  fi_server* s = new (std::nothrow) fi_server;
  if (!s) { set_error("out of host memory"); return FI_ENOMEM_HOST; }
  s->dag = dag;
  serving_info(dag, &s->info);
  if (opts) s->opts = *opts;
  if (s->info.state != 1) { set_error("fi_server_start: the DAG is not loaded"); delete s; return FI_ESTATE; }
  if (!s->info.per_member_inputs) { set_error("fi_server_start: the DAG was not built with per_member_inputs"); delete s; return FI_ESTATE; }
  if (hipGetDevice(&s->device) != hipSuccess) { (void)hipGetLastError(); set_error("fi_server_start: no device"); delete s; return FI_EHIP; }
  const size_t n = (size_t)s->info.n_models;
  s->queue.resize(n);
  s->in_flight.assign(n, 0);
  for (size_t m = 0; m < n; ++m) {
    uint8_t* in = static_cast<uint8_t*>(s->dev_alloc((size_t)(s->info.image_bytes * (uint64_t)s->info.max_batch)));
    uint8_t* ob = static_cast<uint8_t*>(s->dev_alloc((size_t)(s->info.out_bytes[m] * (uint64_t)s->info.max_batch)));
    s->in_buf.push_back(in);
    s->out_buf.push_back(ob);
    if (!in || !ob) { set_error("fi_server_start: device allocation failed"); s->release(); delete s; return FI_ENOMEM_DEVICE; }
  }
  fi_status st;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    st = s->start_workers();
  }
  if (st != FI_OK) { set_error("fi_server_start: no stream"); s->release(); delete s; return st; }
  *out = s;
  return FI_OK;
}

fi_status fi_server_submit(fi_server* s, int32_t member, const void* d_image, void* d_output, uint64_t* ticket) {
  if (!s || !d_image || !d_output || !ticket) { set_error("null argument"); return FI_EINVAL; }
  if (member < 0 || member >= s->info.n_models) { set_error("member %d outside [0, %d)", member, s->info.n_models); return FI_EINVAL; }
  std::lock_guard<std::mutex> lk(s->mu);
  if (s->stopping) { set_error("fi_server_submit: the server is stopping"); return FI_ESTATE; }
  if (s->failed != FI_OK) { set_error("server failed: %s", s->failure.c_str()); return s->failed; }
  if (s->swapping && s->swap_slot == member) { set_error("fi_server_submit: member %d is being swapped", member); return FI_ESTATE; }
  const uint64_t t = s->next_ticket++;
  s->queue[(size_t)member].push_back(Request{t, d_image, d_output, now_ms()});
  s->pending.insert(t);
  *ticket = t;
  // while the workers are away for a swap the request waits in its queue; the new workers find it there
  for (auto& w : s->workers)
    if (w->lane == s->info.lane[(size_t)member]) w->cv.notify_one();
  return FI_OK;
}

fi_status fi_server_wait(fi_server* s, uint64_t ticket) {
  if (!s) { set_error("null server"); return FI_EINVAL; }
  std::unique_lock<std::mutex> lk(s->mu);
  if (ticket == 0 || ticket >= s->next_ticket) { set_error("unknown ticket %llu", (unsigned long long)ticket); return FI_EINVAL; }
  s->cv_done.wait(lk, [&] { return s->pending.count(ticket) == 0 || s->failed != FI_OK; });
  if (s->failed != FI_OK) { set_error("server failed: %s", s->failure.c_str()); return s->failed; }
  return FI_OK;
}

fi_status fi_server_query(fi_server* s, fi_server_stats* st) {
  if (!s || !st) { set_error("null argument"); return FI_EINVAL; }
  std::lock_guard<std::mutex> lk(s->mu);
  st->requests = s->n_requests;
  st->passes = s->n_passes;
  st->max_images_per_pass = s->max_images;
  st->mean_images_per_pass = s->n_passes ? (double)s->n_requests / (double)s->n_passes : 0.0;
  st->mean_latency_ms = s->n_requests ? s->sum_latency_ms / (double)s->n_requests : 0.0;
  st->max_latency_ms = s->max_latency_ms;
  st->busy_ms = s->busy_ms;
  return FI_OK;
}

fi_status fi_server_swap(fi_server* s, int32_t slot, const fi_model_spec* model) {
  if (!s || !model) { set_error("null argument"); return FI_EINVAL; }
  if (slot < 0 || slot >= s->info.n_models) { set_error("slot %d outside [0, %d)", slot, s->info.n_models); return FI_EINVAL; }
  {
    std::unique_lock<std::mutex> lk(s->mu);
    if (s->stopping) { set_error("fi_server_swap: the server is stopping"); return FI_ESTATE; }
    if (s->failed != FI_OK) { set_error("server failed: %s", s->failure.c_str()); return s->failed; }
    if (s->swapping) { set_error("fi_server_swap: another swap is in progress"); return FI_ESTATE; }
    // From here on submissions to the slot are refused; what is queued for it is still served by the
    // outgoing model.  Then every worker leaves after its current pass: the swap re-plans the whole
    // DAG, lanes included.
    s->swapping = true; s->swap_slot = slot;
    s->cv_done.wait(lk, [&] { return (s->queue[(size_t)slot].empty() && s->in_flight[(size_t)slot] == 0) || s->failed != FI_OK; });
    if (s->failed != FI_OK) {   // a worker failed while the slot drained: nothing is swapped, the failure is what the caller gets
      s->swapping = false; s->swap_slot = -1;
      set_error("server failed: %s", s->failure.c_str());
      return s->failed;
    }
    s->regroup = true;
  }
  s->join_workers();
  hipStream_t st0 = nullptr;
  fi_status st = FI_OK;
  std::string why;
  if (hipStreamCreateWithFlags(&st0, hipStreamNonBlocking) != hipSuccess) { (void)hipGetLastError(); st = FI_EHIP; why = "no stream for the swap"; }
  if (st == FI_OK) {
    st = fi_swap_model(s->dag, slot, model, st0);
    if (st != FI_OK) why = fi_last_error();
    else if (hipStreamSynchronize(st0) != hipSuccess) { st = FI_EHIP; why = "hipStreamSynchronize failed after the swap"; }
  }
  if (st0) (void)hipStreamDestroy(st0);
  {
    std::lock_guard<std::mutex> lk(s->mu);
    bool serving = true;
    if (st == FI_OK) {
      ServingInfo now;
      serving_info(s->dag, &now);
      if (now.out_bytes[(size_t)slot] > s->info.out_bytes[(size_t)slot]) {
        uint8_t* bigger = static_cast<uint8_t*>(s->dev_alloc((size_t)(now.out_bytes[(size_t)slot] * (uint64_t)s->info.max_batch)));
        if (bigger) { s->dev_free(s->out_buf[(size_t)slot]); s->out_buf[(size_t)slot] = bigger; }
        else { st = FI_ENOMEM_DEVICE; why = "no device memory for the newcomer's output rows"; s->fail(st, why); serving = false; }
      }
      s->info.out_bytes = now.out_bytes;
      s->info.lane = now.lane;
      s->info.n_lanes = now.n_lanes;
    }
    s->regroup = false;
    if (serving && s->start_workers() != FI_OK) {
      s->fail(FI_EHIP, "no stream for a lane worker");
      if (st == FI_OK) { st = FI_EHIP; why = "no stream for a lane worker"; }
    }
    s->swapping = false; s->swap_slot = -1;
  }
  s->cv_done.notify_all();
  if (st != FI_OK) set_error("%s", why.c_str());
  return st;
}

fi_status fi_server_stop(fi_server* s) {
  if (!s) { set_error("null server"); return FI_EINVAL; }
  {
    std::lock_guard<std::mutex> lk(s->mu);
    s->stopping = true;
  }
  s->join_workers();
  const fi_status st = s->failed;
  if (st != FI_OK) set_error("server failed: %s", s->failure.c_str());
  s->release();
  delete s;
  return st;
}

}  // extern "C"
