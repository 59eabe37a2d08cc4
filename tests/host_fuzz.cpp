// Host-side robustness driver for the planner behind the C ABI (no device is touched).
// Built by tests/test_host_sanitizers.py with AddressSanitizer + UndefinedBehaviorSanitizer from the
// library's host sources; the kernel launcher is replaced by the stub below.  It feeds the entry points
//   * random WELL-FORMED layer graphs (every operator of the ABI, random shapes), which must compile, and
//   * the same graphs with a few fields overwritten by arbitrary values, which must be rejected or
//     accepted with a status -- never a crash, an out-of-range access or undefined arithmetic.
// Usage: host_fuzz <first seed> <count>.  Prints one summary line; exit status 0 when every check held.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "fi_internal.h"

namespace fi {
int launch_kernel(const Launch&, const KArgs&, void*, const std::vector<Desc>&) { return 0; }  // never reached
int static_scratch(void**, uint64_t*) { return 1; }                                                // never reached
}  // namespace fi

namespace {

struct Shape { int c, h, w; };

struct Model {
  std::vector<fi_layer_spec> layers;
  std::vector<Shape> shapes;
  std::vector<uint8_t> blob;
  int in_c = 3, in_h = 16, in_w = 16, dtype = FI_BF16, act_dtype = FI_BF16, output = 0;
  fi_model_spec spec() const {
    fi_model_spec s{};
    s.name = "fuzz"; s.dtype = dtype; s.act_dtype = act_dtype; s.in_c = in_c; s.in_h = in_h; s.in_w = in_w;
    s.n_layers = (int32_t)layers.size(); s.layers = layers.data(); s.output_node = output;
    s.weights_packed = 0; s.weights = blob.data(); s.weight_bytes = blob.size();
    return s;
  }
};

struct Rng {
  std::mt19937_64 g;
  explicit Rng(uint64_t s) : g(s) {}
  int below(int n) { return (int)(g() % (uint64_t)n); }
  int range(int lo, int hi) { return lo + below(hi - lo + 1); }
  bool chance(int pct) { return below(100) < pct; }
  template <class T> T pick(std::initializer_list<T> v) { return *(v.begin() + below((int)v.size())); }
};

// Appends a node and returns its index; the weight offsets are laid out afterwards.
int add(Model& m, int op, int input, Shape out, int cin, int cout, int kh, int kw, int stride, int pad, int act,
        int residual = FI_NO_RESIDUAL, int ceil_mode = 0, int groups = 0, int c_first = 0) {
  fi_layer_spec L{};
  L.op = op; L.input = input; L.residual = residual; L.cin = cin; L.cout = cout; L.kh = kh; L.kw = kw;
  L.stride = stride; L.pad = pad; L.act = act; L.ceil_mode = ceil_mode; L.groups = groups; L.c_first = c_first;
  m.layers.push_back(L);
  m.shapes.push_back(out);
  return (int)m.layers.size() - 1;
}

Shape shape_of(const Model& m, int node) { return node < 0 ? Shape{m.in_c, m.in_h, m.in_w} : m.shapes[(size_t)node]; }

int out_size(int n, int k, int stride, int pad, bool ceil_mode) {
  int o = ceil_mode ? (n + 2 * pad - k + stride - 1) / stride + 1 : (n + 2 * pad - k) / stride + 1;
  if (ceil_mode && (o - 1) * stride >= n + pad) --o;   // the last window starts inside the input or its leading padding
  return o;
}

Model well_formed(Rng& r) {
  Model m;
  m.in_c = r.pick({1, 3, 3, 4, 8});
  m.in_h = r.range(6, 36);
  m.in_w = r.chance(70) ? m.in_h : r.range(6, 36);
  m.dtype = FI_BF16;
  m.act_dtype = r.chance(25) ? FI_F32 : FI_BF16;
  const int want = r.range(1, 22);
  int cur = FI_INPUT;
  for (int step = 0; step < want; ++step) {
    const Shape s = shape_of(m, cur);
    const int act = r.below(7);
    int what = r.below(100);
    if (cur == FI_INPUT && what >= 67) what = 0;   // concat, gate, slice and shuffle do not take the model input directly
    if (what < 45) {   // dense convolution, sometimes grouped / rectangular / with a residual
      int kh = r.pick({1, 1, 3, 3, 3, 5, 7}), kw = kh;
      if (r.chance(15)) { kh = r.pick({1, 3, 7}); kw = kh == 1 ? r.pick({3, 7}) : 1; }
      const int stride = r.chance(25) ? 2 : 1;
      const int pad = r.chance(70) ? (kh > kw ? kh : kw) / 2 : 0;
      const int ph = kh == kw || kh > 1 ? pad : 0, pw = kh == kw || kw > 1 ? pad : 0;
      if (s.h + 2 * ph < kh || s.w + 2 * pw < kw) continue;
      int groups = 0;
      int cout = r.pick({1, 3, 8, 10, 16, 24, 32, 40, 64, 72, 96, 130});
      if (kh == kw && r.chance(20)) {
        groups = r.pick({2, 4, 8});
        if (s.c % groups) groups = 0; else cout = groups * r.range(1, 12);
      }
      const Shape o{cout, (s.h + 2 * ph - kh) / stride + 1, (s.w + 2 * pw - kw) / stride + 1};
      int residual = FI_NO_RESIDUAL;
      if (r.chance(40))
        for (int j = (int)m.layers.size() - 1; j >= 0; --j)
          if (m.shapes[(size_t)j].c == o.c && m.shapes[(size_t)j].h == o.h && m.shapes[(size_t)j].w == o.w) { residual = j; break; }
      cur = add(m, FI_CONV2D, cur, o, s.c, cout, kh, kw, stride, pad, act, residual, 0, groups);
    } else if (what < 55) {               // depthwise
      const int k = r.pick({3, 3, 5}), stride = r.chance(30) ? 2 : 1, pad = k / 2;
      cur = add(m, FI_DWCONV2D, cur, {s.c, (s.h + 2 * pad - k) / stride + 1, (s.w + 2 * pad - k) / stride + 1}, s.c, s.c, k, k,
                stride, pad, act);
    } else if (what < 67) {               // pooling windows
      const bool avg = r.chance(40);
      const int k = r.pick({2, 3}), stride = r.pick({1, 2}), pad = r.chance(50) ? (k - 1) / 2 : 0;
      const bool ceil_mode = !avg && r.chance(40);
      if (s.h + 2 * pad < k || s.w + 2 * pad < k) continue;
      const Shape o{s.c, out_size(s.h, k, stride, pad, ceil_mode), out_size(s.w, k, stride, pad, ceil_mode)};
      if (o.h < 1 || o.w < 1) continue;
      cur = add(m, avg ? FI_AVGPOOL2D : FI_MAXPOOL2D, cur, o, 0, 0, k, k, stride, pad, FI_ACT_NONE, FI_NO_RESIDUAL, ceil_mode);
    } else if (what < 75) {               // concat with an earlier tensor of the same extent
      int other = -1;
      for (int j = (int)m.layers.size() - 1; j >= 0; --j)
        if (j != cur && m.shapes[(size_t)j].h == s.h && m.shapes[(size_t)j].w == s.w) { other = j; break; }
      if (other < 0) continue;
      cur = add(m, FI_CONCAT, cur, {s.c + m.shapes[(size_t)other].c, s.h, s.w}, 0, s.c + m.shapes[(size_t)other].c, 1, 1, 1, 0,
                FI_ACT_NONE, other);
    } else if (what < 83) {               // squeeze-and-excitation gate
      const int sq = add(m, FI_GLOBAL_AVGPOOL, cur, {s.c, 1, 1}, 0, 0, 1, 1, 1, 0, FI_ACT_NONE);
      const int mid = r.range(1, 16);
      const int f1 = add(m, FI_CONV2D, sq, {mid, 1, 1}, s.c, mid, 1, 1, 1, 0, FI_ACT_RELU);
      const int f2 = add(m, FI_CONV2D, f1, {s.c, 1, 1}, mid, s.c, 1, 1, 1, 0, r.chance(50) ? FI_ACT_SIGMOID : FI_ACT_HARDSIGMOID);
      cur = add(m, FI_MUL, cur, s, 0, s.c, 1, 1, 1, 0, FI_ACT_NONE, f2);
    } else if (what < 90) {               // channel slice
      if (s.c < 2) continue;
      const int first = r.below(s.c - 1), count = r.range(1, s.c - first);
      cur = add(m, FI_SLICE, cur, {count, s.h, s.w}, 0, count, 1, 1, 1, 0, FI_ACT_NONE, FI_NO_RESIDUAL, 0, 0, first);
    } else {                              // channel shuffle
      const int groups = r.pick({2, 3, 4});
      if (s.c % groups) continue;
      cur = add(m, FI_SHUFFLE, cur, s, 0, s.c, 1, 1, 1, 0, FI_ACT_NONE, FI_NO_RESIDUAL, 0, groups);
    }
  }
  if (cur == FI_INPUT) cur = add(m, FI_CONV2D, cur, {8, m.in_h, m.in_w}, m.in_c, 8, 1, 1, 1, 0, FI_ACT_RELU);
  if (r.chance(80)) {                     // classifier head
    Shape s = shape_of(m, cur);
    if (r.chance(70)) { cur = add(m, FI_GLOBAL_AVGPOOL, cur, {s.c, 1, 1}, 0, 0, 1, 1, 1, 0, FI_ACT_NONE); s = {s.c, 1, 1}; }
    const int classes = r.pick({1, 10, 37, 1000});
    cur = add(m, FI_FC, cur, {classes, 1, 1}, s.c * s.h * s.w, classes, 1, 1, 1, 0, r.chance(20) ? FI_ACT_RELU : FI_ACT_NONE);
    if (r.chance(30)) cur = add(m, FI_SOFTMAX, cur, {classes, 1, 1}, 0, 0, 1, 1, 1, 0, FI_ACT_NONE);
  }
  m.output = cur;
  // canonical blob: weights [cout][cin/groups][kh][kw] in bf16, bias [cout] in fp32, 16-byte aligned
  uint64_t off = 0;
  for (fi_layer_spec& L : m.layers) {
    if (L.op != FI_CONV2D && L.op != FI_DWCONV2D && L.op != FI_FC) continue;
    const uint64_t per = L.op == FI_DWCONV2D ? 1 : (uint64_t)L.cin / (uint64_t)(L.groups > 1 ? L.groups : 1);
    const uint64_t nw = (uint64_t)L.cout * per * (uint64_t)(L.op == FI_FC ? 1 : L.kh * L.kw);
    L.w_off = off; off += (nw * 2 + 15) / 16 * 16;
    L.b_off = off; off += ((uint64_t)L.cout * 4 + 15) / 16 * 16;
  }
  m.blob.resize((size_t)off);
  for (size_t i = 0; i + 1 < m.blob.size(); i += 2) { m.blob[i] = (uint8_t)r.below(256); m.blob[i + 1] = (uint8_t)(0x3b + r.below(3)); }
  return m;
}

int32_t wild(Rng& r) {
  switch (r.below(8)) {
    case 0: return 0;
    case 1: return -1;
    case 2: return INT32_MAX;
    case 3: return INT32_MIN;
    case 4: return r.range(-70000, 70000);
    case 5: return 1 << r.below(31);
    case 6: return r.range(0, 40);
    default: return (int32_t)r.g();
  }
}

void damage(Model& m, Rng& r) {
  const int hits = r.range(1, 3);
  for (int h = 0; h < hits; ++h) {
    fi_layer_spec& L = m.layers[(size_t)r.below((int)m.layers.size())];
    switch (r.below(18)) {
      case 0: L.op = wild(r); break;
      case 1: L.input = wild(r); break;
      case 2: L.residual = wild(r); break;
      case 3: L.cin = wild(r); break;
      case 4: L.cout = wild(r); break;
      case 5: L.kh = wild(r); break;
      case 6: L.kw = wild(r); break;
      case 7: L.stride = wild(r); break;
      case 8: L.pad = wild(r); break;
      case 9: L.act = wild(r); break;
      case 10: L.ceil_mode = wild(r); break;
      case 11: L.groups = wild(r); break;
      case 12: L.c_first = wild(r); break;
      case 13: L.w_off = r.chance(50) ? r.g() : (uint64_t)m.blob.size() - (uint64_t)r.below(64); break;
      case 14: L.b_off = r.chance(50) ? r.g() : (uint64_t)m.blob.size() - (uint64_t)r.below(64); break;
      case 15: m.output = wild(r); break;
      case 16: (r.chance(50) ? m.in_h : m.in_c) = wild(r); break;
      default: m.in_w = wild(r); break;
    }
  }
}

void* host_alloc(size_t n, void*) { return std::malloc(n ? n : 1); }
void host_free(void* p, void*) { std::free(p); }

int failures = 0;
void check(bool ok, const char* what, uint64_t seed) {
  if (!ok) { std::printf("seed %llu: %s (%s)\n", (unsigned long long)seed, what, fi_last_error()); ++failures; }
}

fi_build_opts options(Rng& r) {
  fi_build_opts o{};
  o.max_batch = r.pick({1, 2, 5, 8, 32});
  o.group_levels = r.chance(80);
  o.load_mode = FI_LOAD_ONE_COPY;
  o.serial_lanes = r.chance(30);
  o.per_member_inputs = r.chance(30);
  o.copy_concats = r.chance(30);
  o.separate_affine = r.chance(30);
  o.pin_alloc = host_alloc; o.pin_free = host_free;   // keeps the build off the HIP runtime
  o.dev_alloc = host_alloc; o.dev_free = host_free;
  return o;
}

// Every entry point that works without a device, on one set of members.
bool exercise(std::vector<Model>& members, Rng& r, uint64_t seed, bool must_compile) {
  std::vector<fi_model_spec> specs;
  for (const Model& m : members) specs.push_back(m.spec());
  fi_build_opts opts = options(r);

  // repository-time packing into a buffer of exactly the reported size (an overrun trips the sanitizer)
  std::vector<std::vector<uint8_t>> packed(members.size());
  bool all_packed = true;
  for (size_t i = 0; i < members.size(); ++i) {
    uint64_t bytes = 0;
    const fi_status st = fi_model_packed_size(&specs[i], &bytes);
    if (must_compile) check(st == FI_OK, "fi_model_packed_size rejected a well-formed model", seed);
    if (st != FI_OK || bytes > (1ull << 30)) { all_packed = false; continue; }
    packed[i].resize((size_t)bytes);
    const fi_status sp = fi_model_pack(&specs[i], packed[i].data(), bytes);
    if (must_compile) check(sp == FI_OK, "fi_model_pack rejected a well-formed model", seed);
    if (sp != FI_OK) all_packed = false;
    if (bytes > 16) check(fi_model_pack(&specs[i], packed[i].data(), bytes - 16) != FI_OK, "fi_model_pack accepted a short buffer", seed);
  }

  fi_dag_info foot{};
  const fi_status sf = fi_footprint(specs.data(), (int32_t)specs.size(), &opts, &foot);
  fi_dag* dag = nullptr;
  const fi_status sb = fi_build_dag(specs.data(), (int32_t)specs.size(), &opts, &dag);
  if (must_compile) check(sb == FI_OK, "fi_build_dag rejected well-formed members", seed);
  check((sb == FI_OK) == (sf == FI_OK), "fi_footprint and fi_build_dag disagree on validity", seed);
  check((sb == FI_OK) == (dag != nullptr), "handle does not match the status", seed);
  if (sb == FI_OK) {
    fi_dag_info info{};
    check(fi_query(dag, &info) == FI_OK, "fi_query failed", seed);
    check(info.device_bytes == foot.device_bytes && info.arena_bytes == foot.arena_bytes && info.act_bytes == foot.act_bytes &&
          info.n_launches == foot.n_launches, "footprint differs from the built DAG", seed);
    check(info.n_models == (int32_t)members.size() && info.state == 0 && info.n_device_allocs == 1, "unexpected dag info", seed);
    int32_t total = 0;
    for (const Model& m : members) total += (int32_t)m.layers.size();
    check(info.n_nodes == total, "node count differs from the specs", seed);
    // introspection, in and out of range
    uint64_t act_end = 0;
    for (int32_t i = -1; i <= info.n_nodes; ++i) {
      fi_node_info ni{};
      const fi_status st = fi_node(dag, i, &ni);
      check((st == FI_OK) == (i >= 0 && i < info.n_nodes), "fi_node range check", seed);
      if (st == FI_OK) {
        check(ni.level >= 1 && ni.level <= info.n_levels && ni.launch >= 0 && ni.launch < info.n_launches, "node level / launch out of range", seed);
        if (!ni.is_output && ni.out_off + ni.out_bytes > act_end) act_end = ni.out_off + ni.out_bytes;
      }
    }
    check(act_end <= info.act_bytes, "a tensor lies outside the activation arena", seed);
    for (int32_t i = -1; i <= info.n_launches; ++i) {
      fi_launch_info li{};
      const fi_status st = fi_launch(dag, i, &li);
      check((st == FI_OK) == (i >= 0 && i < info.n_launches), "fi_launch range check", seed);
      if (st == FI_OK) check(li.n_problems >= 1 && li.n_problems <= FI_MAX_GROUP && li.lane >= 0 && li.lane < info.n_lanes, "launch fields out of range", seed);
    }
    for (int32_t i = -1; i <= info.n_models; ++i) {
      fi_member_info mi{};
      const fi_status st = fi_member(dag, i, &mi);
      check((st == FI_OK) == (i >= 0 && i < info.n_models), "fi_member range check", seed);
      if (st == FI_OK) check(mi.arena_off + mi.packed_bytes <= info.arena_bytes, "member weights outside the arena", seed);
    }
    // calls that need a loaded handle
    void* outs[8] = {};
    check(fi_run(dag, outs, 1, outs, nullptr) == FI_ESTATE, "fi_run on an unloaded handle", seed);
    check(fi_unload(dag) == FI_ESTATE, "fi_unload on an unloaded handle", seed);
    // member swap on the host side: replace a member by a fresh well-formed one of the same input shape
    Model fresh = well_formed(r);
    fresh.in_c = members[0].in_c; fresh.in_h = members[0].in_h; fresh.in_w = members[0].in_w;
    const fi_model_spec fs = fresh.spec();
    const fi_status ss = fi_swap_model(dag, r.below((int)members.size()), &fs, nullptr);
    check(ss == FI_OK || ss == FI_EINVAL || ss == FI_EUNSUPPORTED || ss == FI_EBUDGET, "fi_swap_model status", seed);
    check(fi_swap_model(dag, (int32_t)members.size(), &fs, nullptr) == FI_EINVAL, "fi_swap_model slot range", seed);
    check(fi_query(dag, &info) == FI_OK, "fi_query after swap", seed);
    fi_destroy(dag);

    // partition under a budget between one member's and everybody's footprint
    std::vector<int32_t> group_of(members.size(), -1);
    int32_t n_groups = 0;
    const uint64_t budget = foot.device_bytes / (uint64_t)r.range(1, 3) + 1;
    const fi_status spart = fi_partition(specs.data(), (int32_t)specs.size(), &opts, budget, group_of.data(), &n_groups);
    check(spart == FI_OK || spart == FI_EBUDGET, "fi_partition status", seed);
    if (spart == FI_OK) {
      check(n_groups >= 1 && n_groups <= (int32_t)members.size() && group_of[0] == 0, "fi_partition groups", seed);
      for (size_t i = 1; i < members.size(); ++i)
        check(group_of[i] == group_of[i - 1] || group_of[i] == group_of[i - 1] + 1, "fi_partition order", seed);
    }
    // device-layout members, one copy per member
    if (all_packed) {
      for (size_t i = 0; i < members.size(); ++i) {
        specs[i].weights_packed = 1; specs[i].weights = packed[i].data(); specs[i].weight_bytes = packed[i].size();
      }
      opts.load_mode = FI_LOAD_PER_MODEL;
      fi_dag* d2 = nullptr;
      const fi_status s2 = fi_build_dag(specs.data(), (int32_t)specs.size(), &opts, &d2);
      check(s2 == FI_OK, "fi_build_dag rejected device-layout members", seed);
      if (s2 == FI_OK) {
        fi_dag_info i2{};
        check(fi_query(d2, &i2) == FI_OK && i2.n_h2d_copies == 1 + (int32_t)members.size(), "per-model copy count", seed);
        fi_destroy(d2);
      }
    }
  }
  return sb == FI_OK;
}

}  // namespace

int main(int argc, char** argv) {
  const uint64_t first = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1;
  const int count = argc > 2 ? std::atoi(argv[2]) : 100;
  int compiled = 0, rejected = 0, accepted_damaged = 0;
  for (uint64_t seed = first; seed < first + (uint64_t)count; ++seed) {
    Rng r(seed * 0x9E3779B97F4A7C15ull + 1);
    // members of one DAG share the input shape: the first model fixes it, the others are regenerated to match
    std::vector<Model> members;
    members.push_back(well_formed(r));
    const int n = r.range(1, 4);
    while ((int)members.size() < n) {
      if (r.chance(50)) { members.push_back(members[(size_t)r.below((int)members.size())]); continue; }   // identical architecture: same lane
      Rng sub(r.g());
      Model m = well_formed(sub);
      if (m.in_c == members[0].in_c) { m.in_h = members[0].in_h; m.in_w = members[0].in_w; }
      if (m.in_c != members[0].in_c || m.spec().n_layers == 0) continue;
      members.push_back(std::move(m));
    }
    // a model regenerated at another input size may have become ill-formed: only the first member's own
    // graph is guaranteed, so "must compile" is asserted on sets made of the first member and its copies
    bool pure = true;
    for (size_t i = 1; i < members.size(); ++i)
      if (members[i].layers.size() != members[0].layers.size() ||
          std::memcmp(members[i].layers.data(), members[0].layers.data(), members[0].layers.size() * sizeof(fi_layer_spec)) != 0) pure = false;
    if (exercise(members, r, seed, pure)) ++compiled;
    // the same members with a few fields overwritten
    for (int round = 0; round < 3; ++round) {
      std::vector<Model> bad = members;
      damage(bad[(size_t)r.below((int)bad.size())], r);
      if (exercise(bad, r, seed, false)) ++accepted_damaged; else ++rejected;
    }
  }
  // argument checks of the entry points themselves
  fi_dag* none = nullptr;
  fi_dag_info info{};
  check(fi_build_dag(nullptr, 1, nullptr, &none) == FI_EINVAL, "fi_build_dag(NULL)", 0);
  check(fi_query(nullptr, &info) == FI_EINVAL, "fi_query(NULL)", 0);
  fi_destroy(nullptr);
  std::printf("host_fuzz: %d seeds, %d well-formed sets compiled, %d damaged sets rejected, %d damaged sets still valid, %d failed checks\n",
              count, compiled, rejected, accepted_damaged, failures);
  return failures ? 1 : 0;
}
