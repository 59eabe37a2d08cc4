// Host simulation of the request aggregator for ThreadSanitizer (no device is touched).
// Built by tests/test_host_sanitizers.py from fi_server.cpp alone; the HIP runtime calls and the DAG entry
// points the server uses are replaced below by host stand-ins: "device" memory is host memory, a copy is a
// memcpy, and a lane's pass writes, for every image of its member m, the row {m, first input word, generation of m}.
// Several client threads submit and wait at random while the main thread swaps members; every request must
// come back with the row of its own image and member, whatever batch it travelled in.
// Usage: server_sim <clients> <requests per client>.  Exit status 0 when every row was right.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

#include "fi_internal.h"

namespace {
constexpr int kSimMembers = 3, kSimBatch = 4, kImageWords = 16, kOutWords = 4;
std::atomic<int> generation[kSimMembers];   // bumped by every swap of the member
int lane_of[kSimMembers] = {0, 1, 0};       // members 0 and 2 share a lane; every swap regroups (only while no pass runs)
int n_lanes = 2;
std::atomic<int> lane_busy[kSimMembers];    // a lane never has two passes in flight
std::atomic<long> overlap{0};
std::atomic<long> passes{0}, images{0};
thread_local char err_text[256] = "";
}  // namespace

struct fi_dag { int dummy; };

// ---- stand-ins for the HIP runtime ------------------------------------------------------------------
extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) { *s = reinterpret_cast<hipStream_t>(new int(0)); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { delete reinterpret_cast<int*>(s); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipMalloc(void** p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipGetLastError() { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "simulated"; }
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) { std::memcpy(dst, src, n); return hipSuccess; }

// ---- stand-ins for the DAG entry points ----------------------------------------------------------------
fi_status fi_run_lane(fi_dag*, int32_t lane, const void* const* d_inputs, const int32_t* batches, void* const* d_outputs, void*) {
  ++passes;
  if (lane < 0 || lane >= n_lanes) return FI_EINVAL;
  if (lane_busy[lane].exchange(1) != 0) ++overlap;
  for (int m = 0; m < kSimMembers; ++m) {
    if (lane_of[m] != lane) continue;
    if (batches[m] < 0 || batches[m] > kSimBatch) return FI_EINVAL;
    for (int i = 0; i < batches[m]; ++i) {
      const uint32_t* x = static_cast<const uint32_t*>(d_inputs[m]) + (size_t)i * kImageWords;
      uint32_t* y = static_cast<uint32_t*>(d_outputs[m]) + (size_t)i * kOutWords;
      y[0] = (uint32_t)m; y[1] = x[0]; y[2] = (uint32_t)generation[m].load(); y[3] = x[kImageWords - 1];
      ++images;
    }
  }
  lane_busy[lane].store(0);
  return FI_OK;
}
fi_status fi_swap_model(fi_dag*, int32_t slot, const fi_model_spec* model, void*) {
  if (model->n_layers < 0) { std::snprintf(err_text, sizeof(err_text), "refused"); return FI_EINVAL; }
  ++generation[slot];
  // the newcomer forms a lane of its own or joins another member's, by turns
  const int g = generation[slot].load();
  if (g % 3 == 0) { lane_of[0] = 0; lane_of[1] = 1; lane_of[2] = 2; n_lanes = 3; }
  else if (g % 3 == 1) { lane_of[0] = 0; lane_of[1] = 0; lane_of[2] = 1; n_lanes = 2; }
  else { lane_of[0] = 0; lane_of[1] = 0; lane_of[2] = 0; n_lanes = 1; }
  return FI_OK;
}
const char* fi_last_error(void) { return err_text; }
}  // extern "C"

namespace fi {
int launch_copy_rows(const void* const* src, void* const* dst, int32_t n, uint64_t bytes, void*) {
  for (int32_t i = 0; i < n; ++i) std::memcpy(dst[i], src[i], (size_t)bytes);
  return 0;
}
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::vsnprintf(err_text, sizeof(err_text), fmt, ap);
  va_end(ap);
}
void serving_info(const fi_dag*, ServingInfo* out) {
  out->n_models = kSimMembers; out->max_batch = kSimBatch; out->per_member_inputs = 1; out->state = 1;
  out->image_bytes = kImageWords * 4;
  out->out_bytes.assign(kSimMembers, kOutWords * 4);
  out->lane.assign(lane_of, lane_of + kSimMembers);
  out->n_lanes = n_lanes;
  out->opts = fi_build_opts{};
}
}  // namespace fi

int main(int argc, char** argv) {
  const int clients = argc > 1 ? std::atoi(argv[1]) : 4;
  const int per_client = argc > 2 ? std::atoi(argv[2]) : 2000;
  fi_dag dag{0};
  fi_server* srv = nullptr;
  fi_server_opts opts{50, 0};
  if (fi_server_start(&dag, &opts, &srv) != FI_OK) { std::printf("start failed: %s\n", fi_last_error()); return 1; }
  std::atomic<long> wrong{0}, refused{0};
  std::vector<std::thread> th;
  for (int c = 0; c < clients; ++c)
    th.emplace_back([&, c] {
      std::mt19937 rng(1234 + c);
      struct Pending { uint64_t ticket; int member; uint32_t tag; int gen_lo; std::vector<uint32_t> image, out; };
      std::vector<Pending> open;
      auto settle = [&](Pending& p) {
        if (fi_server_wait(srv, p.ticket) != FI_OK) { ++wrong; return; }
        // the generation is the member's at some moment between submission and completion
        if (p.out[0] != (uint32_t)p.member || p.out[1] != p.tag || p.out[3] != ~p.tag ||
            (int)p.out[2] < p.gen_lo || (int)p.out[2] > generation[p.member].load()) ++wrong;
      };
      for (int r = 0; r < per_client; ++r) {
        Pending p;
        p.member = (int)(rng() % kSimMembers);
        p.tag = (uint32_t)(c * 1000003 + r);
        p.image.assign(kImageWords, 7u); p.image[0] = p.tag; p.image[kImageWords - 1] = ~p.tag;
        p.out.assign(kOutWords, 0xdeadbeefu);
        p.gen_lo = generation[p.member].load();
        open.push_back(std::move(p));
        Pending& q = open.back();
        const fi_status st = fi_server_submit(srv, q.member, q.image.data(), q.out.data(), &q.ticket);
        if (st == FI_ESTATE) { ++refused; open.pop_back(); continue; }   // the member was being swapped
        if (st != FI_OK) { ++wrong; open.pop_back(); continue; }
        if (open.size() >= 1 + rng() % 8) { for (Pending& w : open) settle(w); open.clear(); }
      }
      for (Pending& w : open) settle(w);
    });
  // swaps while the clients run, one of them refused by the DAG
  fi_model_spec good{}, bad{};
  bad.n_layers = -1;
  long swaps = 0;
  for (int k = 0; k < 200; ++k) {
    const fi_status st = fi_server_swap(srv, k % kSimMembers, (k % 17 == 5) ? &bad : &good);
    if ((k % 17 == 5) ? st != FI_EINVAL : st != FI_OK) ++wrong;
    if (st == FI_OK) ++swaps;
    std::this_thread::sleep_for(std::chrono::microseconds(200));
  }
  for (std::thread& t : th) t.join();
  fi_server_stats st{};
  if (fi_server_query(srv, &st) != FI_OK) ++wrong;
  const long served = (long)st.requests;
  if (served + refused.load() != (long)clients * per_client || served != images.load() || (long)st.passes != passes.load()) ++wrong;
  if (st.max_images_per_pass > (uint64_t)kSimMembers * kSimBatch || overlap.load() != 0) ++wrong;
  if (fi_server_stop(srv) != FI_OK) ++wrong;
  std::printf("server_sim: %ld requests served in %ld passes (%.2f per pass), %ld refused during swaps, %ld swaps, %ld wrong\n",
              served, passes.load(), st.mean_images_per_pass, refused.load(), swaps, wrong.load());
  return wrong.load() ? 1 : 0;
}
