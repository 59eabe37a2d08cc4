// C ABI: DAG compilation (Algorithm 1, first loop), arena planning, load / run / unload.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <thread>
#include <tuple>

#include "fi_internal.h"

namespace fi {
const char* last_error();

struct Tensor {           // one stored activation tensor (a node's output, or a staged input)
  int32_t first, last;    // live range in levels, inclusive
  int32_t lane;           // -1: shared by all lanes (staged input)
  uint64_t bytes, off;
};

struct StageTensor {      // a staged (channel-padded, activation-dtype) copy of a caller's input
  int32_t adt;            // activation dtype of the copy
  int32_t cp;             // channel stride of the copy (a member's in_cp: 4 when only convolutions read an RGB-like input)
  int32_t member;         // owner when every member has its own input; -1: shared by every member of this dtype and stride
  int32_t lane;           // -1: shared by all lanes
  int32_t last;           // last level that reads it
  uint64_t off;           // placement in the activation arena
};

struct Member {
  fi_model_spec spec;     // borrowed pointers inside
  ModelPlan plan;
  int32_t node0;          // first global node id
  int32_t lane;           // members of identical architecture share a lane (two lanes when they are many and large)
  int32_t sibling_lanes;  // lanes that run this member's architecture side by side
  int32_t stage;          // index of the staged input this member reads
  uint64_t arena_off;     // placement of the packed blob in the weight arena
};

}  // namespace fi

struct fi_dag {
  fi_build_opts opts{};
  std::vector<fi::Member> members;
  std::vector<fi::Node> nodes;        // global ids; input/residual are global (or -1/-2)
  std::vector<fi::Launch> launches;
  std::vector<fi::Desc> descs;
  int32_t n_levels = 0;
  int32_t n_runs = 0;                 // positions in the launch order (= n_levels unless early levels run in member chunks)
  int32_t wdtype = FI_BF16;
  uint64_t desc_bytes = 0, arena_bytes = 0, act_bytes = 0, workspace_bytes = 0, device_bytes = 0;
  uint64_t image_bytes = 0;           // bytes of the pinned image that a load copies (whole arena, or header only)
  uint64_t image_capacity = 0;        // bytes the pinned allocation holds (a swap may shrink image_bytes, never this)
  std::vector<fi::StageTensor> stages;  // staged inputs: one per activation dtype, or one per member
  uint8_t* image = nullptr;           // pinned host image
  bool gathered = false;              // the image is the whole arena (one copy per load); else the header only, members are copied from their blobs
  int32_t n_loads = 0;                // loads so far (FI_LOAD_AUTO gathers before the second)
  uint8_t* dev = nullptr;             // the one device allocation (LOADED only)
  uint64_t dev_capacity = 0;          // its size: what the plan needed at load plus the swap headroom
  uint64_t last_h2d_bytes = 0;        // bytes and copies of the most recent load or member swap
  int32_t last_h2d_copies = 0;
  hipEvent_t copy_done = nullptr;     // recorded after the latest copy out of the pinned image
  std::atomic<bool> copy_pending{false};   // copy_done may not have completed yet: runs order their stream after it
  int32_t state = 0;
  uint64_t macs = 0;
  // captured launch schedule (use_graph): valid for exactly these call arguments
  int32_t n_lanes = 1;
  std::vector<hipStream_t> lane_streams;   // lanes 1.. (lane 0 runs on the caller's stream)
  std::vector<hipEvent_t> lane_events;     // [0] fork, [l] join of lane l
  hipGraphExec_t gexec = nullptr;
  int32_t g_batch = 0;
  const void* g_input = nullptr;
  std::vector<void*> g_outputs;
  bool capturing = false;             // run_impl is being recorded into a graph: no wait on events from outside it
};

using namespace fi;

namespace {

void* pin_alloc(const fi_build_opts& o, size_t n) {
  if (o.pin_alloc) return o.pin_alloc(n, o.user);
  void* p = nullptr;
  if (hipHostMalloc(&p, n, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  return p;
}
void pin_free(const fi_build_opts& o, void* p) {
  if (!p) return;
  if (o.pin_free) o.pin_free(p, o.user);
  else if (!o.pin_alloc) (void)hipHostFree(p);
}

// Copy with a few host threads: one memcpy stream does not saturate host memory bandwidth.
void parallel_copy(uint8_t* dst, const uint8_t* src, uint64_t n) {
  const uint64_t kMin = 8ull << 20;
  unsigned nt = (unsigned)std::min<uint64_t>(8, n / kMin);
  if (nt <= 1) { std::memcpy(dst, src, (size_t)n); return; }
  std::vector<std::thread> th;
  const uint64_t chunk = (n / nt + 4095) & ~4095ull;
  for (unsigned t = 0; t < nt; ++t) {
    const uint64_t lo = (uint64_t)t * chunk;
    if (lo >= n) break;
    const uint64_t len = std::min(chunk, n - lo);
    th.emplace_back([=] { std::memcpy(dst + lo, src + lo, (size_t)len); });
  }
  for (auto& t : th) t.join();
}

// Tile of the implicit GEMM for one node; `group` = problems of the same shape that will share
// its launch.  Larger tiles re-read less and keep the matrix cores busier, but need enough
// workgroups to cover the 256 compute units.  (Any tile yields the same bits: every output
// element accumulates its reduction in the same order whatever the tile.)
int pick_tile(const Node& n, int max_batch, int group, bool wide) {
  const int64_t M = (int64_t)max_batch * n.Ho * n.Wo;
  auto blocks = [&](int t) { return group * ((M + tile_bm(t) - 1) / tile_bm(t)) * ((n.Co + tile_bn(t) - 1) / tile_bn(t)); };
  // Short reductions stream activations (bandwidth-bound): medium tiles keep more workgroups
  // and loads in flight.  Long reductions are matrix-core-bound: the largest tile re-reads least.
  if (n.Cp == 4) return n.Co <= 64 ? T_128x64 : T_128x128;  // 4-channel input: the two-tap gather exists for these tiles
  if (!wide && n.Co <= 64 && n.Kp > 512 && blocks(T_256x64) >= 256) return T_256x64;  // narrow, long reduction: four waves stacked in M
  const int want = (n.Kp <= 512 || wide) ? T_128x128 : T_256x128;  // fp32-activation members: no 256-row tile
  const int order[4] = {T_256x128, T_128x128, T_128x64, T_64x64};
  bool started = false;
  for (int t : order) {
    if (t == want) started = true;
    if (!started) continue;
    if (tile_bn(t) == 128 && n.Co <= 64) continue;
    if (blocks(t) >= 256 || t == T_64x64) return t;
  }
  return T_64x64;
}

// A grouped convolution on the MFMA path whose column tiles can skip the input channels outside their own
// groups: bf16 activations, and a channel stride that whole 64-element reduction tiles divide.  (Other grouped
// convolutions walk all channels; their packed rows are zero outside the group, so the result is the same.)
bool walks_groups(const Node& n, int adt) {
  return n.kind == K_CONV_MFMA && n.groups > 1 && adt == FI_BF16 && n.Cp % 64 == 0 && n.Cp != 4;
}

// Tile of a group-walking convolution: 64 columns (the narrower the tile, the fewer foreign groups it spans and
// the shorter its reduction), rows as for any problem: the largest that still covers the chip.
int pick_group_tile(const Node& n, int max_batch, int group) {
  const int64_t M = (int64_t)max_batch * n.Ho * n.Wo;
  for (int t : {T_256x64, T_128x64})
    if (group * ((M + tile_bm(t) - 1) / tile_bm(t)) * ((n.Co + 63) / 64) >= 256) return t;
  return T_64x64;
}

const char* kind_name(int kind, int tile) {
  switch (kind) {
    case K_STAGE: return "stage_input";
    case K_CONV_DIRECT: return "conv_direct";
    case K_CONV_MFMA: return tile == T_256x128 ? "conv_mfma_256x128" : tile == T_256x64 ? "conv_mfma_256x64" : (tile == T_128x128 || tile == T_128x128_DEEP) ? "conv_mfma_128x128" : tile == T_128x64 ? "conv_mfma_128x64" : "conv_mfma_64x64";
    case K_DWCONV: return "dwconv";
    case K_MAXPOOL: return "maxpool";
    case K_GAP: return "global_avgpool";
    case K_SOFTMAX: return "softmax";
    case K_FC: return "fc_splitk";
    case K_REDUCE: return "splitk_reduce";
    case K_CONCAT: return "concat";
    case K_AVGPOOL: return "avgpool";
    case K_MUL: return "channel_scale";
    case K_GATHER: return "channel_gather";
    case K_CHAIN: return tile ? "conv_chain3" : "conv_chain2";
    case K_STEM: return (tile & 1) ? "conv_stem_pool" : "conv_stem";
  }
  return "?";
}

uint64_t esize(int dt) { return dt == FI_BF16 ? 2 : 4; }

}  // namespace

extern "C" {

const char* fi_last_error(void) { return fi::last_error(); }
const char* fi_version(void) { return "fusedinf-gfx950 0.1"; }

fi_status fi_model_packed_size(const fi_model_spec* model, uint64_t* bytes) {
  if (!model || !bytes) { set_error("null argument"); return FI_EINVAL; }
  ModelPlan p;
  fi_status st = analyze_model(*model, p);
  if (st != FI_OK) return st;
  *bytes = p.packed_bytes;
  return FI_OK;
}

fi_status fi_model_pack(const fi_model_spec* model, void* dst, uint64_t dst_bytes) {
  if (!model || !dst) { set_error("null argument"); return FI_EINVAL; }
  if (model->weights_packed || !model->weights) { set_error("fi_model_pack needs a canonical blob"); return FI_EINVAL; }
  ModelPlan p;
  fi_status st = analyze_model(*model, p);
  if (st != FI_OK) return st;
  if (dst_bytes < p.packed_bytes) { set_error("destination too small: %llu < %llu", (unsigned long long)dst_bytes, (unsigned long long)p.packed_bytes); return FI_EINVAL; }
  pack_model(*model, p, static_cast<uint8_t*>(dst));
  return FI_OK;
}

// Checks one member against the handle's common dtype / input shape and derives its layout.
static fi_status analyze_member(const fi_build_opts& opts, Member& mb, int32_t m, const fi_model_spec* first) {
  if (!mb.spec.weights) { set_error("model %d: no weights", m); return FI_EINVAL; }
  fi_status st = analyze_model(mb.spec, mb.plan);
  if (st != FI_OK) return st;
  if (mb.spec.weights_packed && mb.spec.weight_bytes < mb.plan.packed_bytes) {
    set_error("model %d: packed blob is %llu bytes, layout needs %llu", m, (unsigned long long)mb.spec.weight_bytes, (unsigned long long)mb.plan.packed_bytes);
    return FI_EINVAL; }
  if (opts.load_mode == FI_LOAD_PER_MODEL && !mb.spec.weights_packed) {
    set_error("FI_LOAD_PER_MODEL needs members in device layout (fi_model_pack)"); return FI_EINVAL; }
  if (first && (mb.spec.dtype != first->dtype || mb.spec.in_c != first->in_c || mb.spec.in_h != first->in_h || mb.spec.in_w != first->in_w)) {
    set_error("model %d: members of one DAG share weight dtype and input shape", m); return FI_EINVAL; }
  for (const Node& n : mb.plan.nodes)
    if ((int64_t)opts.max_batch * n.Ho * n.Wo > INT32_MAX || (int64_t)opts.max_batch * n.H * n.W > INT32_MAX) {
      set_error("model %d node %d: batch %d x %d x %d pixels exceeds the 2^31 rows a launch can index", m, n.index, opts.max_batch,
                n.Ho > n.H ? n.Ho : n.H, n.Wo > n.W ? n.Wo : n.W);
      return FI_EUNSUPPORTED; }
  mb.arena_off = kNone;
  return FI_OK;
}

static fi_status plan_dag(fi_dag* g);

static fi_status build_core(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, bool with_image, fi_dag** out);

fi_status fi_build_dag(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, fi_dag** out) {
  return build_core(models, n, opts, true, out);
}

fi_status fi_footprint(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, fi_dag_info* info) {
  if (!info) { set_error("null info"); return FI_EINVAL; }
  fi_dag* g = nullptr;
  fi_status st = build_core(models, n, opts, false, &g);   // plan only: no pinned image, no weight bytes touched
  if (st != FI_OK) return st;
  st = fi_query(g, info);
  delete g;
  return st;
}

static fi_status build_core(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, bool with_image, fi_dag** out) {
  if (!models || n < 1 || !opts || !out) { set_error("null argument or no models"); return FI_EINVAL; }
  if (opts->max_batch < 1 || opts->max_batch > kMaxBatch) { set_error("max_batch must be in [1, %d]", kMaxBatch); return FI_EINVAL; }
  if (opts->load_mode != FI_LOAD_ONE_COPY && opts->load_mode != FI_LOAD_PER_MODEL && opts->load_mode != FI_LOAD_AUTO) { set_error("bad load_mode"); return FI_EINVAL; }
  if ((opts->pin_alloc == nullptr) != (opts->pin_free == nullptr) || (opts->dev_alloc == nullptr) != (opts->dev_free == nullptr)) {
    set_error("allocator callbacks come in alloc/free pairs"); return FI_EINVAL; }
  std::unique_ptr<fi_dag> g(new (std::nothrow) fi_dag);
  if (!g) { set_error("out of host memory"); return FI_ENOMEM_HOST; }
  g->opts = *opts;
  g->members.resize((size_t)n);

  // ---- per-member analysis; all members share dtype and input shape ----------------
  for (int32_t m = 0; m < n; ++m) {
    Member& mb = g->members[(size_t)m];
    mb.spec = models[m];
    const fi_status st = analyze_member(*opts, mb, m, m ? &models[0] : nullptr);
    if (st != FI_OK) return st;
  }
  fi_status st = plan_dag(g.get());
  if (st != FI_OK) return st;

  if (!with_image) { *out = g.release(); return FI_OK; }

  // ---- pinned image: the bytes fi_load copies ----------------------------------------------
  // FI_LOAD_AUTO: members already in device layout need no image until the handle is loaded a second time
  bool all_packed = true;
  for (const Member& mb : g->members) all_packed = all_packed && mb.spec.weights_packed;
  g->gathered = opts->load_mode == FI_LOAD_ONE_COPY || (opts->load_mode == FI_LOAD_AUTO && !all_packed);
  g->image_bytes = g->gathered ? g->arena_bytes : g->desc_bytes;
  g->image_capacity = g->image_bytes;
  g->image = static_cast<uint8_t*>(pin_alloc(*opts, (size_t)g->image_bytes));
  if (!g->image) { set_error("pinned allocation of %llu bytes failed", (unsigned long long)g->image_bytes); return FI_ENOMEM_HOST; }
  std::memset(g->image, 0, (size_t)g->desc_bytes);
  std::memcpy(g->image, "fusedinf-arena-1", 16);
  if (g->gathered) {
    for (const Member& mb : g->members) {
      if (mb.spec.weights_packed) parallel_copy(g->image + mb.arena_off, static_cast<const uint8_t*>(mb.spec.weights), mb.plan.packed_bytes);
      else pack_model(mb.spec, mb.plan, g->image + mb.arena_off);
    }
  }
  *out = g.release();
  return FI_OK;
}

// Planner pass (kernel families, tiles and split factors are known; launches are not built yet).
static void store_concat_sources_in_place(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t total = (int32_t)g->nodes.size();
  // ---- concatenations in place --------------------------------------------------------------
  // A concatenation copies its two sources into one tensor.  When a source's producer can write with a
  // channel stride other than its own (the MFMA convolution and the bf16 vector kernels can) and whoever
  // else reads that source can read with such a stride (the depthwise kernels can), the source is stored
  // inside the concatenation's tensor from the start and the copy disappears: DenseNet blocks, Inception
  // and fire modules then write every branch once.  Nested concatenations resolve to the outermost tensor.
  for (Node& nd : g->nodes) { nd.root = -1; nd.chan = 0; nd.elided = 0; nd.pre = -1; }
  if (!opts->copy_concats && g->wdtype == FI_BF16) {
    std::vector<std::vector<int32_t>> readers((size_t)total);   // nodes reading a tensor as their first input
    std::vector<int32_t> as_second((size_t)total, 0);           // times a tensor is a second operand (residual, gate, second source)
    for (int32_t i = 0; i < total; ++i) {
      const Node& nd = g->nodes[(size_t)i];
      if (nd.input >= 0) readers[(size_t)nd.input].push_back(i);
      if (nd.residual >= 0) as_second[(size_t)nd.residual]++;
    }
    std::vector<int8_t> can_elide((size_t)total, 0);
    auto stored_in_place = [&](int32_t s, int32_t q, bool second) {
      const Node& S = g->nodes[(size_t)s];
      const int adt = g->members[(size_t)S.model].spec.act_dtype;
      if (adt != FI_BF16 || S.is_output || S.out_dtype != FI_BF16 || S.Cop % 8) return false;
      // the concatenation is the only node that takes S as a second operand (once) or lists it first (once) ...
      if (as_second[(size_t)s] != (second ? 1 : 0)) return false;
      int first_uses = 0;
      for (int32_t r : readers[(size_t)s]) {
        if (r == q) { ++first_uses; continue; }
        if (g->nodes[(size_t)r].kind != K_DWCONV) return false;   // ... and every other reader takes an input stride
      }
      if (first_uses != (second ? 0 : 1)) return false;
      switch (S.kind) {
        case K_CONV_MFMA: return true;
        case K_DWCONV: case K_MAXPOOL: case K_AVGPOOL: case K_GATHER: return S.Cp % 8 == 0;   // their 8-channel forms
        case K_CONCAT: return can_elide[(size_t)s] != 0;
        default: return false;
      }
    };
    for (int32_t i = 0; i < total; ++i) {   // sources come before the concatenation that joins them
      const Node& Q = g->nodes[(size_t)i];
      if (Q.kind != K_CONCAT || Q.input < 0 || Q.residual < 0 || Q.input == Q.residual) continue;
      if (Q.is_output || Q.out_dtype != FI_BF16) continue;   // a model output goes to the caller's buffer: that copy stays
      const Node& A = g->nodes[(size_t)Q.input];
      if (A.Co % 8 || Q.Cop % 8) continue;   // the second source starts on a vector boundary and A has no padding channels
      can_elide[(size_t)i] = stored_in_place(Q.input, i, false) && stored_in_place(Q.residual, i, true);
    }
    for (int32_t i = total - 1; i >= 0; --i) {   // outermost first: an inner concatenation inherits its place
      Node& Q = g->nodes[(size_t)i];
      if (!can_elide[(size_t)i]) continue;
      // an inner concatenation that could be elided but whose outer one cannot still owns its tensor (root stays -1)
      Q.elided = 1;
      const int32_t root = Q.root >= 0 ? Q.root : i;
      Node& A = g->nodes[(size_t)Q.input];
      Node& Bn = g->nodes[(size_t)Q.residual];
      A.root = root; A.chan = Q.chan;
      Bn.root = root; Bn.chan = Q.chan + A.Co;
    }
  }
}

// Planner pass, after store_concat_sources_in_place: nodes that their single reader applies itself.
static void fold_nodes_into_readers(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  // ---- per-channel affine nodes applied by the convolution that reads them -------------------
  // y = act(x * scale[c] + shift[c]) (a 1x1 depthwise node: the normalisation + ReLU in front of a DenseNet
  // layer's 1x1 convolution) read by nothing but one pointwise MFMA convolution: that convolution applies it to
  // its input vectors on their way into LDS, with the arithmetic and the single rounding of the depthwise
  // kernel, so the bits are the same and the node needs neither a launch nor a tensor.
  if (!opts->separate_affine && g->wdtype == FI_BF16) {
    std::vector<int32_t> n_readers((size_t)total, 0), only_reader((size_t)total, -1);
    for (int32_t i = 0; i < total; ++i) {
      const Node& nd = g->nodes[(size_t)i];
      if (nd.input >= 0) { n_readers[(size_t)nd.input]++; only_reader[(size_t)nd.input] = i; }
      if (nd.residual >= 0) n_readers[(size_t)nd.residual] += 2;   // a second operand: never fused
    }
    for (int32_t i = 0; i < total; ++i) {
      Node& A = g->nodes[(size_t)i];
      const int adt = g->members[(size_t)A.model].spec.act_dtype;
      if (A.kind != K_DWCONV || A.k != 1 || A.stride != 1 || A.pad != 0 || A.residual >= 0 || A.input < 0) continue;
      if (adt != FI_BF16 || A.is_output || A.out_dtype != FI_BF16 || A.root >= 0) continue;
      if (!(A.act == FI_ACT_NONE || A.act == FI_ACT_RELU || A.act == FI_ACT_RELU6)) continue;   // act(0) = 0 keeps padding channels zero
      if (n_readers[(size_t)i] != 1) continue;
      Node& V = g->nodes[(size_t)only_reader[(size_t)i]];
      if (V.kind != K_CONV_MFMA || V.k != 1 || V.kw != 1 || V.stride != 1 || V.pad != 0 || V.pad_w != 0) continue;
      if (V.groups > 1 || V.Cp == 4 || V.Cp != A.Cp) continue;
      const Node& T = g->nodes[(size_t)A.input];
      if (T.out_dtype != FI_BF16) continue;
      const int64_t stride = T.root >= 0 ? g->nodes[(size_t)T.root].Cop : T.Cop;
      if ((uint64_t)B * V.H * V.W * (uint64_t)stride * 2 >= (1ull << 31)) continue;   // the conv kernel's 32-bit byte offsets
      V.pre = i;
      A.elided = 1;
    }
    // y = x * gate[image][c] (the scaling that ends a squeeze-excite block) read by nothing but one pointwise MFMA
    // convolution (the block's projection): the convolution multiplies its input vectors by the gate on their way
    // into LDS, with the scaling kernel's fp32 product and single rounding.
    for (int32_t i = 0; i < total; ++i) {
      Node& Y = g->nodes[(size_t)i];
      const int adt = g->members[(size_t)Y.model].spec.act_dtype;
      if (Y.kind != K_MUL || Y.input < 0 || Y.residual < 0 || Y.is_output || Y.out_dtype != adt || Y.root >= 0) continue;   // (bf16 or fp32 tensors)
      if (n_readers[(size_t)i] != 1) continue;
      Node& V = g->nodes[(size_t)only_reader[(size_t)i]];
      if (V.kind != K_CONV_MFMA || V.k != 1 || V.kw != 1 || V.stride != 1 || V.pad != 0 || V.pad_w != 0 || V.pre >= 0) continue;
      if (V.groups > 1 || V.Cp == 4 || V.Cp != Y.Cop || V.Cp % 8) continue;
      const Node& T = g->nodes[(size_t)Y.input];
      const Node& G = g->nodes[(size_t)Y.residual];
      if (T.out_dtype != adt || G.out_dtype != adt || G.is_output || G.root >= 0 || G.Cop != V.Cp) continue;
      const int64_t stride = T.root >= 0 ? g->nodes[(size_t)T.root].Cop : T.Cop;
      if ((uint64_t)B * V.H * V.W * (uint64_t)stride * esize(adt) >= (1ull << 31)) continue;
      V.pre = i;
      Y.elided = 1;
    }
    // shuffle_2(concat(A, B)) with equal halves (the end of a ShuffleNet unit) read by nothing else: the shuffle
    // interleaves A and B itself and the concatenation is never built.  (A concatenation already stored in place
    // costs nothing and stays.)
    for (int32_t i = 0; i < total; ++i) {
      Node& Z = g->nodes[(size_t)i];
      if (Z.kind != K_GATHER || Z.op != FI_SHUFFLE || Z.k != 2 || Z.input < 0) continue;
      Node& Q = g->nodes[(size_t)Z.input];
      if (Q.kind != K_CONCAT || Q.elided || Q.root >= 0 || Q.is_output || n_readers[(size_t)Z.input] != 1 || Q.input < 0 || Q.residual < 0) continue;
      const Node& A = g->nodes[(size_t)Q.input];
      const Node& Bn = g->nodes[(size_t)Q.residual];
      if (A.Co != Bn.Co || A.out_dtype != Q.out_dtype || Bn.out_dtype != Q.out_dtype || A.root >= 0 || Bn.root >= 0) continue;
      Z.pre = Z.input;
      Q.elided = 2;   // never built: no launch and no tensor
    }
  }
}

// Planner pass, after fold_nodes_into_readers: chains of convolutions that one launch carries through.
// A dense convolution A (bf16 in and out, 64 or 128 output channels, whole 64-element reduction tiles per filter tap)
// whose ONLY reader is a pointwise convolution B (any multiple of 128 output channels, optional residual), and
// optionally a pointwise convolution C that reads B (64 or 128 output channels, no residual): a workgroup that owns
// 128 output pixels of A finishes the same pixels of B and C.  A's output is stored nowhere, B's and C's are written
// as ever.  In a ResNet bottleneck stage: A = a block's 3x3, B = its 1x1 expansion with the shortcut added,
// C = the next block's 1x1 reduction (or the next stage's first one).
static void form_chains(fi_dag* g) {
  const int32_t total = (int32_t)g->nodes.size();
  for (Node& nd : g->nodes) { nd.chain = -1; nd.chain_pos = 0; }
  if (g->opts.separate_chains || g->wdtype != FI_BF16) return;
  std::vector<std::vector<int32_t>> readers((size_t)total);   // nodes reading a tensor as their first input
  std::vector<int32_t> other_uses((size_t)total, 0);          // uses as a second operand, or by a node fused into its reader
  for (int32_t i = 0; i < total; ++i) {
    const Node& nd = g->nodes[(size_t)i];
    if (nd.input >= 0) readers[(size_t)nd.input].push_back(i);
    if (nd.residual >= 0) other_uses[(size_t)nd.residual]++;
  }
  auto plain_conv = [&](const Node& n) {   // a dense bf16 MFMA convolution with nothing folded into or around it
    const int adt = g->members[(size_t)n.model].spec.act_dtype;
    return n.kind == K_CONV_MFMA && n.op == FI_CONV2D && adt == FI_BF16 && n.out_dtype == FI_BF16 && n.groups == 1 && n.pre < 0 && n.root < 0 &&
           !n.elided && !n.is_output && n.splits == 1 && n.Cp != 4 && n.chain < 0;
  };
  auto pointwise = [](const Node& n) { return n.k == 1 && n.kw == 1 && n.stride == 1 && n.pad == 0 && n.pad_w == 0; };
  for (int32_t i = 0; i < total; ++i) {
    Node& A = g->nodes[(size_t)i];
    if (!plain_conv(A) || A.residual >= 0 || A.Cp % 64 || A.C != A.Cp || (A.Co != 64 && A.Co != 128) || A.Co != A.Cop) continue;
    if (A.Kp != A.k * A.kw * A.Cp || A.input < 0) continue;
    if (A.input >= 0 && g->nodes[(size_t)A.input].root >= 0) continue;   // an input inside a concatenation has a pixel stride of its own
    if (readers[(size_t)i].size() != 1 || other_uses[(size_t)i] != 0) continue;
    const int32_t bi = readers[(size_t)i][0];
    Node& Bn = g->nodes[(size_t)bi];
    if (!plain_conv(Bn) || !pointwise(Bn) || Bn.level != A.level + 1 || Bn.run != A.run + 1 || Bn.C != A.Co || Bn.Cp != A.Cop || Bn.Co % 128 || Bn.Co > 1024 || Bn.Co != Bn.Cop || Bn.Kp != Bn.Cp) continue;
    // the chained launch addresses B's rows (and 127 past the last) with 32-bit byte offsets
    if (((uint64_t)g->opts.max_batch * A.Ho * A.Wo + 128) * (uint64_t)Bn.Cop * 2 >= (1ull << 31)) continue;
    if (Bn.residual >= 0) {
      const Node& R = g->nodes[(size_t)Bn.residual];
      if (R.root >= 0 || R.out_dtype != FI_BF16 || R.Cop != Bn.Cop || Bn.residual == i) continue;
      if (R.run >= A.run) continue;   // the chain runs in A's place: everything it reads is complete by then
    }
    int32_t ci = -1;
    for (int32_t r : readers[(size_t)bi]) {
      const Node& Cn = g->nodes[(size_t)r];
      if (!plain_conv(Cn) || !pointwise(Cn) || Cn.residual >= 0 || Cn.level != Bn.level + 1 || Cn.run != Bn.run + 1) continue;
      if (Cn.C != Bn.Co || Cn.Cp != Bn.Cop || Cn.Kp != Cn.Cp || (Cn.Co != 64 && Cn.Co != 128) || Cn.Co != Cn.Cop) continue;
      ci = r;
      break;
    }
    A.chain = i; A.chain_pos = 0;
    Bn.chain = i; Bn.chain_pos = 1; Bn.run = A.run;
    if (ci >= 0) { g->nodes[(size_t)ci].chain = i; g->nodes[(size_t)ci].chain_pos = 2; g->nodes[(size_t)ci].run = A.run; }
    A.tile = ci >= 0 ? 1 : 0;   // (the chained launch has no tile choice: the field tells chains of three from chains of two)
  }
}

// Planner pass, after form_chains: the first convolution of an ImageNet-style member.  A 7x7 stride-2, 3x3 stride-1 or 3x3
// stride-2 convolution over the 4-channel model input with 64 output channels (bf16 in and out, identity / ReLU / ReLU6) takes the stem kernel, which
// multiplies from an input patch in LDS instead of gathering reduction vectors from memory.  When its ONLY reader is a
// 3x3 stride-2 max-pool (padding 0 or 1, floor or ceil mode), that pool is part of the same launch: the pool node carries the launch,
// the convolution gets none and its output is stored nowhere.  Same bits as the general kernels either way.
static void take_stem_launches(fi_dag* g) {
  if (g->opts.separate_stem || g->wdtype != FI_BF16) return;
  const int32_t total = (int32_t)g->nodes.size();
  const uint64_t B = (uint64_t)g->opts.max_batch;
  std::vector<int32_t> uses((size_t)total, 0);   // readers of a tensor, as first or second operand
  for (const Node& nd : g->nodes) {
    if (nd.input >= 0) uses[(size_t)nd.input]++;
    if (nd.residual >= 0) uses[(size_t)nd.residual]++;
  }
  for (Node& A : g->nodes) {
    const int adt = g->members[(size_t)A.model].spec.act_dtype;
    if (A.kind != K_CONV_MFMA || A.op != FI_CONV2D || adt != FI_BF16 || A.out_dtype != FI_BF16 || A.input >= 0 || A.residual >= 0) continue;
    const int geom = stem_geometry(A.k, A.kw, A.stride);
    if (A.Cp != 4 || geom < 0 || A.pad < 0 || A.pad > A.k / 2 || A.pad_w < 0 || A.pad_w > A.k / 2) continue;
    if (A.H + 2 * A.pad < A.k || A.W + 2 * A.pad_w < A.k) continue;
    if (A.Co != 64 || A.Cop != 64 || A.Kp != (A.k * A.k * 4 + 31) / 32 * 32 || A.groups != 1 || A.act > FI_ACT_RELU6) continue;
    if (A.is_output || A.root >= 0 || A.elided || A.pre >= 0 || A.chain >= 0 || A.splits != 1) continue;
    if (B * A.Ho * A.Wo * 64 * 2 >= (1ull << 31)) continue;   // the kernel's 32-bit output offsets
    A.kind = K_STEM;
    A.tile = 2 * geom;
  }
  for (int32_t i = 0; i < total; ++i) {
    Node& P = g->nodes[(size_t)i];
    if (P.kind != K_MAXPOOL || P.input < 0 || P.k != 3 || P.stride != 2 || P.pad < 0 || P.pad > 1) continue;
    Node& A = g->nodes[(size_t)P.input];
    if (A.kind != K_STEM || A.stride != 2 || uses[(size_t)P.input] != 1) continue;
    if (P.is_output || P.elided || P.out_dtype != FI_BF16 || P.Cp != 64 || P.Cop != 64 || P.run != A.run + 1) continue;
    // (the pooled tensor may be stored inside a concatenation's, as the first tensor of a DenseNet block is: the launch writes
    // it at that tensor's pixel stride, which has to stay within the kernel's 32-bit offsets)
    if (P.root >= 0 && B * P.Ho * P.Wo * (uint64_t)g->nodes[(size_t)P.root].Cop * 2 >= (1ull << 31)) continue;
    // floor or ceil mode: all the kernel needs is that every window starts inside the convolution's output
    if ((P.Ho - 1) * 2 - P.pad >= A.Ho || (P.Wo - 1) * 2 - P.pad >= A.Wo) continue;
    P.pre = P.input;
    P.kind = K_STEM;
    P.tile = A.tile | 1;
    A.elided = 1;
  }
}

// Planner pass, after the passes that fold nodes into convolutions: a plain bf16 convolution on the 128x128 tile whose
// reduction is long (32 tiles or more) and whose member brings few workgroups (64 at most: with eight members a launch
// still has at most two per compute unit) keeps three reduction tiles in flight in registers instead of one.  Such a
// launch has nothing else to hide a load behind; the deeper prefetch costs registers that launches of many workgroups
// need for residency, so they keep the plain tile.  (The summation order, hence every bit, is the same.)
static void deepen_long_reductions(fi_dag* g) {
  if (g->wdtype != FI_BF16) return;
  const int64_t B = g->opts.max_batch;
  for (Node& nd : g->nodes) {
    const int adt = g->members[(size_t)nd.model].spec.act_dtype;
    if (nd.kind != K_CONV_MFMA || nd.tile != T_128x128 || adt != FI_BF16 || nd.out_dtype != FI_BF16) continue;
    if (nd.pre >= 0 || nd.elided || nd.chain >= 0 || nd.splits != 1 || nd.Cp == 4 || walks_groups(nd, adt)) continue;
    const int64_t blocks = ((B * nd.Ho * nd.Wo + 127) / 128) * ((nd.Co + 127) / 128);
    if (nd.Kp >= 32 * 64 && blocks <= 64) nd.tile = T_128x128_DEEP;
  }
}

// Planner pass: the disjoint union of the member graphs and every node's depth.
static void union_member_graphs(fi_dag* g) {
  const int32_t n = (int32_t)g->members.size();
  // ---- union of the member graphs (no edge between members) and depth levels --------
  int32_t total = 0;
  for (auto& mb : g->members) { mb.node0 = total; total += (int32_t)mb.plan.nodes.size(); }
  g->nodes.reserve((size_t)total);
  for (int32_t m = 0; m < n; ++m) {
    const Member& mb = g->members[(size_t)m];
    for (const Node& ln : mb.plan.nodes) {
      Node gn = ln;
      gn.model = m;
      if (gn.input >= 0) gn.input += mb.node0;
      if (gn.residual >= 0) gn.residual += mb.node0;
      int32_t lv = gn.input >= 0 ? g->nodes[(size_t)gn.input].level : 0;
      if (gn.residual >= 0) lv = std::max(lv, g->nodes[(size_t)gn.residual].level);
      gn.level = lv + 1;
      g->n_levels = std::max(g->n_levels, gn.level);
      g->macs += gn.macs;
      g->nodes.push_back(gn);
    }
  }

}

// Planner pass: members of one architecture share a lane; large families are halved.
static void assign_lanes(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- lanes: members whose graphs are identical node for node share launches level by level;
  //      members of different architecture rarely do, so each architecture gets a lane of its
  //      own that runs concurrently with the others (no edge joins two members).  A large family
  //      of large members is halved into two lanes: every launch of a half still covers the chip,
  //      and the tail of one lane's launch (workgroups draining, stores in flight, the next launch
  //      starting up) is filled by the other lane's work instead of idling. --------------------
  {
    std::map<std::string, std::vector<int32_t>> family;   // architecture signature -> members, in order
    std::vector<std::string> order;
    for (size_t mi = 0; mi < g->members.size(); ++mi) {
      Member& mb = g->members[mi];
      std::string sig = std::to_string(mb.spec.act_dtype);
      for (const Node& n : mb.plan.nodes) {
        char buf[96];
        std::snprintf(buf, sizeof(buf), "|%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", n.op, n.input, n.residual, n.C, n.Co, n.k, n.kw, n.stride, n.pad, n.act);
        sig += buf;
      }
      if (!family.count(sig)) order.push_back(sig);
      family[sig].push_back((int32_t)mi);
    }
    int32_t next_lane = 0;
    for (const std::string& sig : order) {
      const std::vector<int32_t>& mem = family[sig];
      const int32_t m = (int32_t)mem.size();
      // halve when most convolutions of half the family still give every compute unit a 128x128 tile
      int32_t convs = 0, full = 0;
      for (const Node& n : g->members[(size_t)mem[0]].plan.nodes) {
        if (n.op != FI_CONV2D) continue;
        ++convs;
        const int64_t tiles = (((int64_t)opts->max_batch * n.Ho * n.Wo + 127) / 128) * ((n.Co + 127) / 128);
        if (tiles * (m / 2) >= 256) ++full;
      }
      const int32_t halves = (!opts->serial_lanes && m >= 4 && convs > 0 && 2 * full >= convs) ? 2 : 1;
      for (int32_t j = 0; j < m; ++j) {
        Member& mb = g->members[(size_t)mem[(size_t)j]];
        mb.lane = opts->serial_lanes ? 0 : next_lane + (halves == 2 && j >= (m + 1) / 2 ? 1 : 0);
        mb.sibling_lanes = halves;
      }
      next_lane += halves;
    }
    g->n_lanes = opts->serial_lanes ? 1 : next_lane;
    for (Node& nd : g->nodes) nd.lane = g->members[(size_t)nd.model].lane;
  }

}

// Planner pass: the position of every node in the launch order (its depth, or shifted when early levels run in member chunks).
static void assign_run_positions(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- launch order: by depth, except that the early levels of a lane may run in member chunks --------
  for (Node& nd : g->nodes) nd.run = nd.level;
  g->n_runs = g->n_levels;
  if (opts->member_chunks >= 2) {
    // Per lane (its members have one architecture): the depth S after which a member's live activations stay below
    // two thirds of their peak.  Levels 1..S run chunk by chunk (chunk k shifted by k S), everything deeper after
    // the last chunk.  A shift common to a whole lane changes nothing between lanes: they are not level-synchronous.
    int32_t longest = g->n_levels;
    for (int32_t lane = 0; lane < g->n_lanes; ++lane) {
      std::vector<int32_t> mem;
      for (int32_t m = 0; m < n; ++m) if (g->members[(size_t)m].lane == lane) mem.push_back(m);
      const int32_t chunks = std::min<int32_t>(opts->member_chunks, (int32_t)mem.size());
      if (chunks < 2) continue;
      const Member& first = g->members[(size_t)mem[0]];
      const int32_t nn = (int32_t)first.plan.nodes.size();
      std::vector<int32_t> last((size_t)nn);
      std::vector<uint64_t> live((size_t)g->n_levels + 2, 0);
      for (int32_t i = 0; i < nn; ++i) last[(size_t)i] = g->nodes[(size_t)(first.node0 + i)].level;
      for (int32_t i = 0; i < nn; ++i) {
        const Node& nd = g->nodes[(size_t)(first.node0 + i)];
        if (nd.input >= 0) last[(size_t)(nd.input - first.node0)] = std::max(last[(size_t)(nd.input - first.node0)], nd.level);
        if (nd.residual >= 0) last[(size_t)(nd.residual - first.node0)] = std::max(last[(size_t)(nd.residual - first.node0)], nd.level);
      }
      for (int32_t i = 0; i < nn; ++i) {
        const Node& nd = g->nodes[(size_t)(first.node0 + i)];
        const uint64_t bytes = nd.is_output ? 0 : (uint64_t)B * nd.Ho * nd.Wo * nd.Cop * esize(nd.out_dtype);
        for (int32_t lv = nd.level; lv <= last[(size_t)i]; ++lv) live[(size_t)lv] += bytes;
      }
      uint64_t peak = 0;
      for (uint64_t v : live) peak = std::max(peak, v);
      int32_t S = 0;
      for (int32_t lv = g->n_levels; lv >= 1; --lv)
        if (live[(size_t)lv] * 3 > peak * 2) { S = lv; break; }
      if (S <= 0 || S >= g->n_levels) continue;
      const int32_t per = ((int32_t)mem.size() + chunks - 1) / chunks;
      for (size_t j = 0; j < mem.size(); ++j) {
        const Member& mb = g->members[(size_t)mem[j]];
        const int32_t k = (int32_t)j / per;
        for (size_t t = 0; t < mb.plan.nodes.size(); ++t) {
          Node& nd = g->nodes[(size_t)mb.node0 + t];
          nd.run = nd.level <= S ? nd.level + k * S : nd.level + (chunks - 1) * S;
        }
      }
      longest = std::max(longest, g->n_levels + (chunks - 1) * S);
    }
    g->n_runs = longest;
  }

}

// Planner pass: kernel family, tile and reduction split of every node.
static fi_status choose_kernels(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- kernel family per node ---------------------------------------------------------
  std::map<std::tuple<int, int, int, int, int, int>, int> same_shape;  // problems of one shape per level
  for (const Node& nd : g->nodes)
    if (nd.op == FI_CONV2D || nd.op == FI_FC) same_shape[std::make_tuple(nd.run + 10000 * nd.lane, nd.Ho * nd.Wo, nd.Co, nd.Kp, nd.k, nd.stride)]++;
  for (Node& nd : g->nodes) {
    const int adt = g->members[(size_t)nd.model].spec.act_dtype;
    nd.tile = 0;
    switch (nd.op) {
      case FI_CONV2D:
      case FI_FC:
        if (g->wdtype == FI_BF16 && nd.op == FI_FC) {
          // a weight stream: 32 images fill one MFMA column block, larger batches take one pass per 32 images
          nd.kind = K_FC;
          const int tiles = (nd.Co + 31) / 32, steps = nd.Kp / 16;
          nd.splits = std::max(1, std::min(std::min(64, std::max(1, steps / 8)), std::max(1, 2048 / tiles)));
          if (nd.Kp <= 512) nd.splits = 1;   // a short reduction (a squeeze-excite gate, a small head): the kernel finishes it itself
          // A split layer with a small weight matrix (latency-bound: a gate, a classifier head) keeps all slices of a
          // tile in one workgroup, which sums them in LDS and finishes: no partials in HBM, no reduce launch.
          if (nd.splits > 1 && nd.splits <= 16 && (uint64_t)((nd.Co + 31) / 32 * 32) * (uint64_t)nd.Kp * 2 <= (4u << 20)) nd.tile = 1;
        } else if (g->wdtype == FI_BF16) {
          nd.kind = K_CONV_MFMA;
          {
            // Small problems cannot cover the chip and walk a long serial reduction: split K.  The split
            // count depends on the node's own shape only (it fixes the summation order, and a member's bits
            // must not depend on its co-members).
            const int64_t M = (int64_t)B * nd.Ho * nd.Wo;
            const int64_t nb64 = ((M + 63) / 64) * ((nd.Co + 63) / 64);
            const int ntiles = (nd.Kp + 63) / 64;
            nd.splits = nd.Cp == 4 ? 1 : (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(16, ntiles / 4), 256 / nb64));
            if (ntiles < 16) nd.splits = 1;   // a reduction under 1024 elements is over before the extra reduce launch would pay
          }
          // the kernel addresses its input with 32-bit byte offsets through a buffer resource
          if ((uint64_t)B * nd.Ho * nd.Wo >= (1ull << 24)) {  // row indices are decoded with exact float arithmetic
            set_error("model %d node %d: more than 2^24 output pixels per launch", nd.model, nd.index);
            return FI_EUNSUPPORTED;
          }
          if ((uint64_t)B * nd.H * nd.W * nd.Cp * esize(adt) >= (1ull << 31)) {
            set_error("model %d node %d: input tensor of %llu bytes exceeds the 2 GiB a conv kernel addresses",
                      nd.model, nd.index, (unsigned long long)((uint64_t)B * nd.H * nd.W * nd.Cp * esize(adt)));
            return FI_EUNSUPPORTED;
          }
          const int grp = opts->group_levels ? same_shape[std::make_tuple(nd.run + 10000 * nd.lane, nd.Ho * nd.Wo, nd.Co, nd.Kp, nd.k, nd.stride)] : 1;
          // sibling lanes run the same level at about the same time: the chip is shared by all of them
          nd.tile = pick_tile(nd, B, std::min(grp * g->members[(size_t)nd.model].sibling_lanes, (int)FI_MAX_GROUP), adt == FI_F32);
          if (walks_groups(nd, adt)) {   // the reduction shrinks to the tile's own groups: short, never split
            nd.tile = pick_group_tile(nd, B, std::min(grp * g->members[(size_t)nd.model].sibling_lanes, (int)FI_MAX_GROUP));
            nd.splits = 1;
          }
        } else nd.kind = K_CONV_DIRECT;
        break;
      case FI_DWCONV2D: nd.kind = K_DWCONV; break;
      case FI_MAXPOOL2D: nd.kind = K_MAXPOOL; break;
      case FI_GLOBAL_AVGPOOL: nd.kind = K_GAP; break;
      case FI_CONCAT: nd.kind = K_CONCAT; break;
      case FI_AVGPOOL2D: nd.kind = K_AVGPOOL; break;
      case FI_MUL: nd.kind = K_MUL; break;
      case FI_SLICE:
      case FI_SHUFFLE: nd.kind = K_GATHER; break;
      default: nd.kind = K_SOFTMAX; break;
    }
  }

  return FI_OK;
}

// Planner pass: staged inputs and the launch list: per position, nodes of one family, tile and storage dtypes share a launch.
static void build_schedule(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- launch schedule: per level, nodes of one family (and tile, and storage dtypes)
  //      share a launch, FI_MAX_GROUP problems at most --------------------------------------
  // staged inputs: the shared input once per activation dtype, or every member's own input
  if (opts->per_member_inputs) {
    for (int32_t m = 0; m < n; ++m) {
      Member& mb = g->members[(size_t)m];
      mb.stage = (int32_t)g->stages.size();
      g->stages.push_back(StageTensor{mb.spec.act_dtype, mb.plan.in_cp, m, g->n_lanes > 1 ? mb.lane : -1, 0, 0});
    }
  } else {
    // one copy per (activation dtype, channel stride) that some member reads
    for (Member& mb : g->members) {
      const int adt = mb.spec.act_dtype;
      mb.stage = -1;
      for (size_t t = 0; t < g->stages.size(); ++t)
        if (g->stages[t].adt == adt && g->stages[t].cp == mb.plan.in_cp) mb.stage = (int32_t)t;
      if (mb.stage < 0) { mb.stage = (int32_t)g->stages.size(); g->stages.push_back(StageTensor{adt, mb.plan.in_cp, -1, -1, 0, 0}); }
    }
  }
  auto new_launch = [&](int level, int kind, int tile, int adt) -> Launch& {
    Launch L{};
    L.level = level; L.kind = kind; L.tile = tile; L.wdtype = g->wdtype; L.adtype = adt; L.lane = 0;
    L.first_desc = 0; L.n = 0; L.macs = L.act_bytes = L.weight_bytes = 0;
    L.name = kind_name(kind, tile);
    g->launches.push_back(L);
    return g->launches.back();
  };
  for (int adt = 0; adt < 2; ++adt) {
    int32_t open_stage = -1;
    for (size_t t = 0; t < g->stages.size(); ++t) {
      if (g->stages[t].adt != adt) continue;
      if (open_stage < 0 || g->launches[(size_t)open_stage].n >= FI_MAX_GROUP) {
        new_launch(0, K_STAGE, 0, adt);
        open_stage = (int32_t)g->launches.size() - 1;
      }
      Launch& L = g->launches[(size_t)open_stage];
      L.nodes.push_back((int32_t)t);   // a staging launch lists staged tensors, not nodes
      ++L.n;
    }
  }
  for (int32_t lv = 1; lv <= g->n_runs; ++lv) {
    std::map<std::tuple<int, int, int>, int32_t> open;   // (kind, tile, adtype/split/lane) -> launch index
    for (int32_t i = 0; i < total; ++i) {
      Node& nd = g->nodes[(size_t)i];
      if (nd.run != lv) continue;
      if (nd.elided) {   // a concatenation in place is complete once its second source is written: reported under that launch
        nd.launch = nd.kind == K_CONCAT ? g->nodes[(size_t)nd.residual].launch : 0;   // (a fused affine node: set below)
        nd.slot = 0;
        continue;
      }
      if (nd.chain >= 0 && nd.chain_pos > 0) continue;   // runs inside its chain's launch (set when the head is scheduled)
      if (nd.chain == i) {
        // the head of a chain: one problem = the chain's two or three nodes; launches are shared by chains of one shape
        int32_t bi = -1, ci = -1;
        for (int32_t r = i + 1; r < total; ++r) {
          const Node& f = g->nodes[(size_t)r];
          if (f.chain != i) continue;
          if (f.chain_pos == 1) bi = r; else if (f.chain_pos == 2) ci = r;
        }
        const int shape = nd.Co * 4 + (ci >= 0 ? g->nodes[(size_t)ci].Co / 64 : 0);   // the kernel's template arguments
        const auto key = std::make_tuple((int)K_CHAIN, shape, nd.lane);
        auto it = open.find(key);
        if (!opts->group_levels || it == open.end() || g->launches[(size_t)it->second].n + 3 > FI_MAX_GROUP) {
          new_launch(lv, K_CHAIN, ci >= 0 ? 1 : 0, FI_BF16).lane = nd.lane;
          open[key] = (int32_t)g->launches.size() - 1;
          it = open.find(key);
        }
        Launch& L = g->launches[(size_t)it->second];
        const int32_t trio[3] = {i, bi, ci >= 0 ? ci : bi};   // (a chain of two repeats its second node in the third place)
        for (int t3 = 0; t3 < 3; ++t3) {
          Node& f = g->nodes[(size_t)trio[t3]];
          if (t3 < 2 || ci >= 0) { f.launch = it->second; f.slot = L.n; }
          L.nodes.push_back(trio[t3]);
          ++L.n;
        }
        continue;
      }
      const int adt = g->members[(size_t)nd.model].spec.act_dtype;
      const int pre_kind = (nd.pre < 0 || nd.kind == K_STEM) ? 0 : g->nodes[(size_t)nd.pre].kind == K_MUL ? 2 : 1;
      const auto key = std::make_tuple(nd.kind, nd.tile, nd.lane * 64 + pre_kind * 16 + (walks_groups(nd, adt) ? 8 : 0) + (nd.kind == K_CONV_MFMA && nd.Cp == 4 ? 4 : 0) + adt * 2 +
                                       ((nd.kind == K_CONV_MFMA || nd.kind == K_FC) && nd.splits > 1 ? 1 : 0));
      auto it = open.find(key);
      if (!opts->group_levels || it == open.end() || g->launches[(size_t)it->second].n >= FI_MAX_GROUP) {
        new_launch(lv, nd.kind, nd.tile, adt).lane = nd.lane;
        open[key] = (int32_t)g->launches.size() - 1;
        it = open.find(key);
      }
      Launch& L = g->launches[(size_t)it->second];
      nd.launch = it->second;
      nd.slot = L.n++;
      L.nodes.push_back(i);
    }
    // every split-K FC launch is followed by the launch that reduces its partials
    const size_t level_end = g->launches.size();
    for (size_t li = 0; li < level_end; ++li) {
      const Launch& cand = g->launches[li];
      const bool split_conv = cand.kind == K_CONV_MFMA && !cand.nodes.empty() && g->nodes[(size_t)cand.nodes[0]].splits > 1;
      if (cand.level != lv || !(cand.kind == K_FC || split_conv)) continue;
      if (cand.kind == K_FC) {   // FC launches whose problems are all unsplit finish in their own kernel
        bool any_split = false;
        for (int32_t ni : cand.nodes) any_split = any_split || g->nodes[(size_t)ni].splits > 1;
        if (!any_split || cand.tile == 1) continue;   // (tile 1: the FC kernel that sums its slices itself)
      }
      const Launch src = cand;
      Launch& R = new_launch(lv, K_REDUCE, 0, src.adtype);
      R.lane = src.lane;
      R.n = src.n;
      R.nodes = src.nodes;
    }
  }

  for (const Node& nd : g->nodes)
    if (nd.pre >= 0) { g->nodes[(size_t)nd.pre].launch = nd.launch; g->nodes[(size_t)nd.pre].slot = nd.slot; }

}

// Planner pass: live range of every stored tensor (in launch-order positions), then first fit by size.
static void plan_activation_arena(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- activation arena: live range of every stored tensor, then first-fit by size -----
  const int32_t n_stage = (int32_t)g->stages.size();
  std::vector<Tensor> tens((size_t)total + (size_t)n_stage);
  for (int32_t i = 0; i < total; ++i) {
    Node& nd = g->nodes[(size_t)i];
    nd.first_level = nd.last_level = nd.run;   // (live ranges are counted in launch order)
  }
  for (int32_t i = 0; i < total; ++i) {
    const Node& nd = g->nodes[(size_t)i];
    if (nd.input >= 0) g->nodes[(size_t)nd.input].last_level = std::max(g->nodes[(size_t)nd.input].last_level, nd.run);
    else { StageTensor& st = g->stages[(size_t)g->members[(size_t)nd.model].stage]; st.last = std::max(st.last, nd.run); }
    if (nd.residual >= 0) g->nodes[(size_t)nd.residual].last_level = std::max(g->nodes[(size_t)nd.residual].last_level, nd.run);
    if (nd.pre >= 0 && g->nodes[(size_t)nd.pre].input < 0) {   // a stem launch with its pool reads the staged model input
      StageTensor& st = g->stages[(size_t)g->members[(size_t)nd.model].stage];
      st.last = std::max(st.last, nd.run);
    } else if (nd.pre >= 0) {   // the convolution reads the fused node's input (and gate) itself
      Node& T = g->nodes[(size_t)g->nodes[(size_t)nd.pre].input];
      T.last_level = std::max(T.last_level, nd.run);
      if (g->nodes[(size_t)nd.pre].kind == K_MUL || g->nodes[(size_t)nd.pre].kind == K_CONCAT) {
        Node& G = g->nodes[(size_t)g->nodes[(size_t)nd.pre].residual];
        G.last_level = std::max(G.last_level, nd.run);
      }
    }
  }
  for (int32_t i = 0; i < total; ++i) {   // a tensor stored inside a concatenation lives in that node's buffer
    const Node& nd = g->nodes[(size_t)i];
    if (nd.root < 0) continue;
    Node& R = g->nodes[(size_t)nd.root];
    R.first_level = std::min(R.first_level, nd.first_level);
    R.last_level = std::max(R.last_level, nd.last_level);
  }
  for (int32_t i = 0; i < total; ++i) {
    Node& nd = g->nodes[(size_t)i];
    nd.out_bytes = (nd.is_output || nd.root >= 0 || (nd.elided && nd.kind != K_CONCAT) || nd.elided == 2 || nd.chain == i) ? 0 : align_up((uint64_t)B * nd.Ho * nd.Wo * nd.Cop * esize(nd.out_dtype));
    tens[(size_t)i] = Tensor{nd.first_level, nd.last_level, nd.lane, nd.out_bytes, 0};
  }
  const Member& m0 = g->members[0];
  for (int32_t t = 0; t < n_stage; ++t) {
    const StageTensor& st = g->stages[(size_t)t];
    tens[(size_t)(total + t)] = Tensor{0, st.last, st.lane,
        align_up((uint64_t)B * m0.spec.in_h * m0.spec.in_w * st.cp * esize(st.adt)), 0};
  }
  {
    std::vector<int32_t> order;
    for (int32_t i = 0; i < total + n_stage; ++i) if (tens[(size_t)i].bytes) order.push_back(i);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return tens[(size_t)a].bytes > tens[(size_t)b].bytes; });
    std::vector<int32_t> placed;
    uint64_t top = 0;
    for (int32_t t : order) {
      Tensor& T = tens[(size_t)t];
      // offsets blocked by tensors alive at the same time, scanned in address order
      std::vector<std::pair<uint64_t, uint64_t>> busy;
      for (int32_t u : placed) {
        const Tensor& U = tens[(size_t)u];
        // lanes are not level-synchronous with each other: tensors of different lanes never share memory
        const bool other_lane = g->n_lanes > 1 && (U.lane != T.lane || U.lane < 0);
        if (other_lane || (U.first <= T.last && T.first <= U.last)) busy.emplace_back(U.off, U.off + U.bytes);
      }
      std::sort(busy.begin(), busy.end());
      uint64_t off = 0;
      for (auto& b : busy) { if (off + T.bytes <= b.first) break; off = std::max(off, b.second); }
      T.off = off;
      top = std::max(top, off + T.bytes);
      placed.push_back(t);
    }
    g->act_bytes = align_up(top ? top : kAlign);
  }
  for (int32_t i = 0; i < total; ++i) g->nodes[(size_t)i].out_off = tens[(size_t)i].off;
  for (int32_t i = 0; i < total; ++i) {
    Node& nd = g->nodes[(size_t)i];
    if (nd.root >= 0) nd.out_off = g->nodes[(size_t)nd.root].out_off + (uint64_t)nd.chan * esize(nd.out_dtype);
  }
  for (int32_t t = 0; t < n_stage; ++t) g->stages[(size_t)t].off = tens[(size_t)(total + t)].off;

}

// Planner pass: members in the weight arena, split-K partials in the workspace, the budget check.
static fi_status place_weights_and_workspace(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  // ---- weight arena: [descriptor table][member 0][member 1]... --------------------------
  size_t n_desc = 0;
  for (Launch& L : g->launches) { L.first_desc = (int32_t)n_desc; n_desc += (size_t)L.n; }
  g->descs.assign(n_desc, Desc{});
  g->desc_bytes = kAlign;  // arena header; problem descriptors travel as launch arguments
  {
    std::vector<std::pair<uint64_t, uint64_t>> used;   // resident members, in address order
    for (const Member& mb : g->members)
      if (mb.arena_off != kNone) used.emplace_back(mb.arena_off, mb.arena_off + mb.plan.packed_bytes);
    for (Member& mb : g->members) {
      if (mb.arena_off != kNone) continue;
      std::sort(used.begin(), used.end());
      uint64_t off = g->desc_bytes;
      for (const auto& u : used) { if (off + mb.plan.packed_bytes <= u.first) break; off = std::max(off, u.second); }
      mb.arena_off = off;
      used.emplace_back(off, off + mb.plan.packed_bytes);
    }
    uint64_t top = g->desc_bytes;
    for (const auto& u : used) top = std::max(top, u.second);
    g->arena_bytes = align_up(top);
  }
  for (Node& nd : g->nodes) {
    const Member& mb = g->members[(size_t)nd.model];
    nd.w_off = nd.w_rel == kNone ? kNone : mb.arena_off + nd.w_rel;
    nd.b_off = nd.b_rel == kNone ? kNone : mb.arena_off + nd.b_rel;
  }
  // workspace: split-K partials; nodes of one level get disjoint regions, levels reuse them
  g->workspace_bytes = 0;
  {
    // per lane: nodes of one level get disjoint regions, levels reuse them; lanes never share
    std::vector<uint64_t> lane_need((size_t)g->n_lanes, 0);
    std::map<std::pair<int32_t, int32_t>, uint64_t> level_top;
    for (Node& nd : g->nodes) {
      if (!(nd.kind == K_FC || (nd.kind == K_CONV_MFMA && nd.splits > 1))) continue;
      uint64_t& top = level_top[{nd.lane, nd.run}];
      nd.ws_off = top;
      top += align_up((uint64_t)nd.splits * B * nd.Ho * nd.Wo * nd.Cop * 4);
      lane_need[(size_t)nd.lane] = std::max(lane_need[(size_t)nd.lane], top);
    }
    std::vector<uint64_t> lane_base((size_t)g->n_lanes, 0);
    for (int32_t l = 0; l < g->n_lanes; ++l) { lane_base[(size_t)l] = g->workspace_bytes; g->workspace_bytes += lane_need[(size_t)l]; }
    for (Node& nd : g->nodes)
      if (nd.kind == K_FC || (nd.kind == K_CONV_MFMA && nd.splits > 1)) nd.ws_off += lane_base[(size_t)nd.lane];
  }
  g->device_bytes = g->arena_bytes + g->act_bytes + g->workspace_bytes;
  if (opts->max_device_bytes && g->device_bytes > opts->max_device_bytes) {
    set_error("DAG needs %llu device bytes, budget is %llu", (unsigned long long)g->device_bytes, (unsigned long long)opts->max_device_bytes);
    return FI_EBUDGET;
  }

  return FI_OK;
}

// Planner pass: one problem descriptor per launch slot, and the per-launch work accounting.
static void fill_descriptors(fi_dag* g) {
  const fi_build_opts* opts = &g->opts;
  const int32_t n = (int32_t)g->members.size();
  const int32_t total = (int32_t)g->nodes.size();
  const int B = opts->max_batch;
  (void)opts; (void)n; (void)total; (void)B;
  const Member& m0 = g->members[0];
  // ---- descriptors ---------------------------------------------------------------------
  for (Launch& L : g->launches) {
    if (L.kind == K_STAGE) {
      for (int32_t k = 0; k < L.n; ++k) {
        Desc& d = g->descs[(size_t)(L.first_desc + k)];
        d.H = m0.spec.in_h; d.W = m0.spec.in_w; d.C = m0.spec.in_c; d.Cp = g->stages[(size_t)L.nodes[(size_t)k]].cp;
        d.y_off = g->stages[(size_t)L.nodes[(size_t)k]].off; d.r_off = kNone; d.x_off = d.w_off = d.b_off = kNone;
        L.act_bytes += (uint64_t)d.H * d.W * (d.C * esize(L.wdtype) + d.Cp * esize(L.adtype));
      }
      continue;
    }
    for (int32_t s = 0; s < L.n; ++s) {
      const Node& nd = g->nodes[(size_t)L.nodes[(size_t)s]];
      const int adt = g->members[(size_t)nd.model].spec.act_dtype;
      Desc& d = g->descs[(size_t)(L.first_desc + s)];
      if (L.kind == K_STEM) {   // the convolution's fields (the node itself, or the one in front of the pool that carries the launch)
        const Node& cv = (L.tile & 1) ? g->nodes[(size_t)nd.pre] : nd;
        d.x_off = g->stages[(size_t)g->members[(size_t)nd.model].stage].off;
        d.y_off = nd.out_off;
        d.r_off = d.pw_off = d.pb_off = kNone;
        d.w_off = cv.w_off; d.b_off = cv.b_off;
        d.H = cv.H; d.W = cv.W; d.C = cv.C; d.Cp = cv.Cp; d.xs = cv.Cp;
        d.k = cv.k; d.kw = cv.kw; d.stride = cv.stride; d.pad = cv.pad; d.pad_w = cv.pad_w; d.act = cv.act; d.Kp = cv.Kp;
        d.gin = cv.Ho; d.gout = cv.Wo;
        d.pre_act = (L.tile & 1) ? nd.pad : 0;   // (with the pool: its padding)
        d.Ho = nd.Ho; d.Wo = nd.Wo; d.Co = nd.Co; d.Cop = nd.Cop;
        d.ys = nd.root >= 0 ? g->nodes[(size_t)nd.root].Cop : nd.Cop;
        d.splits = 1;
        d.ws_off = kNone;
        // workgroups walk several pixel blocks: as many as stay resident together (two per compute unit), over the launch's
        // problems and the lanes that run the same level at about the same time
        d.tiles_n = std::max(16, 512 / std::max(1, L.n * g->members[(size_t)nd.model].sibling_lanes));
        L.macs += cv.macs;
        L.act_bytes += (uint64_t)cv.H * cv.W * cv.C * 2 + (uint64_t)nd.Ho * nd.Wo * nd.Co * 2;
        L.weight_bytes += (uint64_t)cv.Co * cv.k * cv.kw * cv.C * 2 + (uint64_t)cv.Co * 4;
        continue;
      }
      d.x_off = nd.input >= 0 ? g->nodes[(size_t)nd.input].out_off : g->stages[(size_t)g->members[(size_t)nd.model].stage].off;
      d.y_off = nd.is_output ? kNone : nd.out_off;
      d.r_off = nd.residual >= 0 ? g->nodes[(size_t)nd.residual].out_off : kNone;
      d.w_off = nd.w_off; d.b_off = nd.b_off;
      d.H = nd.H; d.W = nd.W; d.C = nd.C; d.Cp = nd.Cp;
      d.Ho = nd.Ho; d.Wo = nd.Wo; d.Co = nd.Co; d.Cop = nd.Cop;
      d.k = nd.k; d.stride = nd.stride; d.pad = nd.pad; d.act = nd.act; d.Kp = nd.Kp;
      d.kw = nd.kw; d.pad_w = nd.pad_w;
      if (nd.op == FI_SLICE) d.stride = 0;     // gather mode: slice
      if (nd.op == FI_SHUFFLE) d.stride = 1;   // gather mode: shuffle
      if (nd.op == FI_CONCAT) {  // second source: channels in Kp, channel stride in tiles_n (set below)
        d.Kp = g->nodes[(size_t)nd.residual].Co;
      }
      if (nd.op == FI_FC) {  // a fully connected node is a 1x1 convolution over the flattened input
        d.C = d.Cp = nd.H * nd.W * nd.Cp; d.H = d.W = 1; d.k = d.kw = 1; d.stride = 1; d.pad = d.pad_w = 0;
      }
      d.ext = nd.is_output;
      d.vec = (adt == FI_BF16 && nd.Cp % 8 == 0 && nd.Cop % 8 == 0 && !nd.is_output && nd.out_dtype == FI_BF16) ? 1 : 0;
      d.out_f32 = (nd.out_dtype == FI_F32 && adt != FI_F32) ? 1 : 0;
      if (nd.out_dtype == FI_F32 && adt != FI_F32 && !nd.is_output) d.Cop = nd.Cop;  // fp32 rows keep the padded stride
      d.tiles_n = L.kind == K_CONV_MFMA ? (nd.Co + tile_bn(L.tile) - 1) / tile_bn(L.tile) : 0;
      d.splits = std::max(1, nd.splits);
      if (walks_groups(nd, adt)) { d.gin = nd.C / nd.groups; d.gout = nd.Co / nd.groups; }
      {
        const Node* in = nd.input >= 0 ? &g->nodes[(size_t)nd.input] : nullptr;
        d.pw_off = d.pb_off = kNone;
        if (nd.pre >= 0 && g->nodes[(size_t)nd.pre].kind == K_CONCAT) {   // a shuffle that interleaves the concatenation's two sources
          const Node& Q = g->nodes[(size_t)nd.pre];
          const Node& A = g->nodes[(size_t)Q.input];
          const Node& Bn = g->nodes[(size_t)Q.residual];
          in = &A;
          d.x_off = A.out_off; d.r_off = Bn.out_off;
          d.Cp = A.Cop; d.tiles_n = Bn.Cop; d.stride = 2;
          d.vec = (d.vec && A.Cop % 8 == 0 && Bn.Cop % 8 == 0) ? 1 : 0;
        } else if (nd.pre >= 0) {   // read the affine node's input, apply the node on the way in
          const Node& A = g->nodes[(size_t)nd.pre];
          in = &g->nodes[(size_t)A.input];
          d.x_off = in->out_off;
          if (A.kind == K_MUL) { d.pre_kind = 2; d.pw_off = g->nodes[(size_t)A.residual].out_off; }
          else { d.pre_kind = 1; d.pw_off = A.w_off; d.pb_off = A.b_off; d.pre_act = A.act; }
        }
        d.xs = (in && in->root >= 0) ? g->nodes[(size_t)in->root].Cop : d.Cp;
        d.ys = nd.root >= 0 ? g->nodes[(size_t)nd.root].Cop : d.Cop;
      }
      d.ws_off = nd.ws_off;  // relative to the workspace (which follows the activation arena in a loaded handle)
      if (L.kind == K_FC) d.tiles_n = (nd.Co + 31) / 32;
      if (L.kind == K_CONCAT) {
        const Node& second = g->nodes[(size_t)nd.residual];
        d.tiles_n = second.Cop;
        d.vec = (d.vec && nd.C % 8 == 0 && second.Cop % 8 == 0) ? 1 : 0;  // whole 8-channel vectors come from one source
      }
      if (L.kind == K_REDUCE) {
        L.act_bytes += ((uint64_t)nd.splits * nd.Cop * 4 + (uint64_t)nd.Co * esize(nd.out_dtype)) * nd.Ho * nd.Wo;
        continue;
      }
      if (L.kind == K_CHAIN && s % 3 == 2 && L.nodes[(size_t)s] == L.nodes[(size_t)s - 1]) continue;   // the filler of a chain of two
      L.macs += nd.macs;
      const uint64_t in_e = esize(nd.input >= 0 ? g->nodes[(size_t)nd.input].out_dtype : adt);
      if (L.kind == K_CHAIN)   // the head's input, the second node's residual and output, the third node's output: nothing in between
        L.act_bytes += (s % 3 == 0 ? (uint64_t)nd.H * nd.W * nd.C * in_e : (uint64_t)nd.Ho * nd.Wo * nd.Co * esize(nd.out_dtype)) +
                       (nd.residual >= 0 ? (uint64_t)nd.Ho * nd.Wo * nd.Co * esize(adt) : 0);
      else
      L.act_bytes += (uint64_t)nd.H * nd.W * nd.C * in_e + (uint64_t)nd.Ho * nd.Wo * nd.Co * esize(nd.out_dtype) +
                     (nd.residual >= 0 ? (uint64_t)nd.Ho * nd.Wo * nd.Co * esize(adt) : 0);
      if (nd.w_rel != kNone)
        L.weight_bytes += (nd.op == FI_DWCONV2D ? (uint64_t)nd.k * nd.k * nd.C : (uint64_t)nd.Co * nd.k * nd.k * nd.C * (nd.op == FI_FC ? nd.H * nd.W : 1)) * esize(g->wdtype) + (uint64_t)nd.Co * 4;
    }
  }

  // pooling launches whose problems are all 3x3 stride-1 windows on bf16 vectors run the strip kernel
  // (4 neighbouring outputs per thread; the strip length travels in the otherwise unused tiles_n)
  for (Launch& L : g->launches) {
    if (L.kind != K_MAXPOOL && L.kind != K_AVGPOOL) continue;
    bool strip = L.adtype == FI_BF16;
    for (int32_t s = 0; s < L.n; ++s) {
      const Desc& d = g->descs[(size_t)(L.first_desc + s)];
      strip = strip && d.vec && d.k == 3 && d.stride == 1 && !d.ext;
    }
    for (int32_t s = 0; s < L.n; ++s) g->descs[(size_t)(L.first_desc + s)].tiles_n = strip ? 4 : 0;
  }

  // depthwise / global-average launches use the 8-channel vector kernels only when every problem allows it
  for (Launch& L : g->launches) {
    if (L.kind != K_DWCONV && L.kind != K_GAP) continue;
    bool vec = L.kind == K_GAP || g->wdtype == FI_BF16;
    for (int32_t s = 0; s < L.n; ++s) {
      const Desc& d = g->descs[(size_t)(L.first_desc + s)];
      vec = vec && d.Cp % 8 == 0 && d.Cop % 8 == 0;
    }
    for (int32_t s = 0; s < L.n; ++s) g->descs[(size_t)(L.first_desc + s)].vec = vec ? 1 : 0;
    // A depthwise launch whose problems all have the same 3x3 / 5x5 / 7x7 filter and stride 1 or 2 runs the
    // strip kernel: a thread computes 4 (stride 1) or 2 (stride 2) neighbouring outputs of a row from one
    // pass over the input pixels they share.  The strip length travels in the (otherwise unused) tiles_n.
    if (L.kind == K_DWCONV) {
      const Desc& d0 = g->descs[(size_t)L.first_desc];
      bool strip = vec && (d0.k == 3 || d0.k == 5 || d0.k == 7) && (d0.stride == 1 || d0.stride == 2);
      for (int32_t s = 1; s < L.n; ++s) {
        const Desc& d = g->descs[(size_t)(L.first_desc + s)];
        strip = strip && d.k == d0.k && d.stride == d0.stride;
      }
      for (int32_t s = 0; s < L.n; ++s) g->descs[(size_t)(L.first_desc + s)].tiles_n = strip ? (d0.stride == 1 ? 4 : 2) : 1;
    }
  }

}

// Everything derived from the member list: union graph, levels, lanes, kernels and tiles, launch
// schedule, activation plan, weight arena placement, workspace, descriptors.  Members whose
// arena_off is already set keep their place in the weight arena (their bytes may be resident);
// the others go to the lowest gap that holds them.
static fi_status plan_dag(fi_dag* g) {
  g->nodes.clear(); g->launches.clear(); g->descs.clear();
  g->n_levels = 0; g->macs = 0; g->n_lanes = 1;
  g->stages.clear();
  g->wdtype = g->members[0].spec.dtype;
  union_member_graphs(g);
  assign_lanes(g);
  assign_run_positions(g);
  fi_status st = choose_kernels(g);
  if (st != FI_OK) return st;
  // nodes that need no launch of their own: concatenations written in place, nodes applied by their reader, chains
  store_concat_sources_in_place(g);
  fold_nodes_into_readers(g);
  form_chains(g);
  take_stem_launches(g);
  deepen_long_reductions(g);
  build_schedule(g);
  plan_activation_arena(g);
  st = place_weights_and_workspace(g);
  if (st != FI_OK) return st;
  fill_descriptors(g);
  return FI_OK;
}

fi_status fi_query(const fi_dag* g, fi_dag_info* info) {
  if (!g || !info) { set_error("null argument"); return FI_EINVAL; }
  std::memset(info, 0, sizeof(*info));
  info->arena_bytes = g->arena_bytes; info->act_bytes = g->act_bytes; info->workspace_bytes = g->workspace_bytes;
  info->device_bytes = g->device_bytes; info->macs_per_image = g->macs;
  info->n_models = (int32_t)g->members.size(); info->n_nodes = (int32_t)g->nodes.size();
  info->n_levels = g->n_levels; info->n_launches = (int32_t)g->launches.size();
  info->n_device_allocs = 1;
  info->n_h2d_copies = g->gathered ? 1 : 1 + (int32_t)g->members.size();
  info->state = g->state;
  info->n_lanes = g->n_lanes;
  info->device_capacity = g->dev_capacity;
  info->last_h2d_bytes = g->last_h2d_bytes;
  info->last_h2d_copies = g->last_h2d_copies;
  if (!g->members.empty()) {
    const fi_model_spec& m0 = g->members[0].spec;
    info->input_image_bytes = (uint64_t)m0.in_h * m0.in_w * m0.in_c * esize(m0.dtype);
  }
  return FI_OK;
}

fi_status fi_node(const fi_dag* g, int32_t i, fi_node_info* o) {
  if (!g || !o || i < 0 || i >= (int32_t)g->nodes.size()) { set_error("bad node index"); return FI_EINVAL; }
  const Node& n = g->nodes[(size_t)i];
  std::memset(o, 0, sizeof(*o));
  o->model = n.model; o->index = n.index; o->op = n.op; o->level = n.level; o->launch = n.launch;
  o->out_c = n.Co; o->out_h = n.Ho; o->out_w = n.Wo; o->out_cp = n.Cop; o->out_dtype = n.out_dtype;
  o->is_output = n.is_output; o->first_level = n.first_level; o->last_level = n.last_level;
  o->out_off = n.out_off; o->out_bytes = n.out_bytes; o->w_off = n.w_off; o->b_off = n.b_off; o->macs = n.macs;
  return FI_OK;
}

fi_status fi_member(const fi_dag* g, int32_t m, fi_member_info* o) {
  if (!g || !o || m < 0 || m >= (int32_t)g->members.size()) { set_error("bad member index"); return FI_EINVAL; }
  const Member& mb = g->members[(size_t)m];
  std::memset(o, 0, sizeof(*o));
  o->arena_off = mb.arena_off; o->packed_bytes = mb.plan.packed_bytes;
  o->lane = mb.lane; o->first_node = mb.node0; o->n_nodes = (int32_t)mb.plan.nodes.size();
  for (const Node& nd : g->nodes)
    if (nd.model == m && nd.is_output) o->output_row_bytes = (uint64_t)nd.Ho * nd.Wo * nd.Co * 4;
  return FI_OK;
}

fi_status fi_launch(const fi_dag* g, int32_t i, fi_launch_info* o) {
  if (!g || !o || i < 0 || i >= (int32_t)g->launches.size()) { set_error("bad launch index"); return FI_EINVAL; }
  const Launch& L = g->launches[(size_t)i];
  std::memset(o, 0, sizeof(*o));
  o->lane = L.lane;
  o->level = L.level; o->kind = L.kind; o->n_problems = L.n;
  o->first_node = (L.nodes.empty() || L.kind == K_STAGE) ? -1 : L.nodes[0];
  o->macs_per_image = L.macs; o->bytes_per_image = L.act_bytes; o->weight_bytes = L.weight_bytes;
  std::snprintf(o->name, sizeof(o->name), "%s", L.name.c_str());
  return FI_OK;
}

// internal streams (default priority) and events for the concurrent lanes; all or nothing
static void ensure_lanes(fi_dag* g) {
  while ((int32_t)g->lane_streams.size() < g->n_lanes - 1) {
    hipStream_t ls = nullptr;
    if (hipStreamCreateWithFlags(&ls, hipStreamNonBlocking) != hipSuccess) { (void)hipGetLastError(); return; }
    g->lane_streams.push_back(ls);
  }
  while ((int32_t)g->lane_events.size() < g->n_lanes) {
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); return; }
    g->lane_events.push_back(ev);
  }
}

// The whole arena image in pinned memory, from a handle that so far held the header only (all members are in device
// layout).  On failure the handle keeps copying member by member.
static bool gather_image(fi_dag* g) {
  uint8_t* whole = static_cast<uint8_t*>(pin_alloc(g->opts, (size_t)g->arena_bytes));
  if (!whole) return false;
  if (g->copy_done) (void)hipEventSynchronize(g->copy_done);   // (the header may still be on its way out of the old image)
  std::memset(whole, 0, (size_t)g->desc_bytes);
  std::memcpy(whole, g->image, (size_t)std::min(g->desc_bytes, g->image_capacity));
  for (const Member& mb : g->members) parallel_copy(whole + mb.arena_off, static_cast<const uint8_t*>(mb.spec.weights), mb.plan.packed_bytes);
  pin_free(g->opts, g->image);
  g->image = whole;
  g->image_capacity = g->image_bytes = g->arena_bytes;
  g->gathered = true;
  return true;
}

fi_status fi_load(fi_dag* g, void* stream) {
  if (!g) { set_error("null handle"); return FI_EINVAL; }
  if (g->state != 0) { set_error("fi_load: handle is already loaded"); return FI_ESTATE; }
  if (g->opts.load_mode == FI_LOAD_AUTO && !g->gathered && g->n_loads > 0) (void)gather_image(g);   // loaded again: worth one image from now on
  const uint64_t want = g->device_bytes + g->opts.swap_headroom_bytes;
  // what the load copies is the plan's arena (or its header), not whatever the pinned allocation can hold:
  // a member swap may have left the plan smaller than the image once was
  const uint64_t copy_bytes = g->gathered ? g->arena_bytes : g->desc_bytes;
  if (copy_bytes > want || copy_bytes > g->image_capacity) {
    set_error("fi_load: the arena image (%llu bytes) does not fit the pinned image (%llu) or the device allocation (%llu)",
              (unsigned long long)copy_bytes, (unsigned long long)g->image_capacity, (unsigned long long)want);
    return FI_ESTATE;
  }
  uint8_t* d = nullptr;
  if (g->opts.dev_alloc) d = static_cast<uint8_t*>(g->opts.dev_alloc((size_t)want, g->opts.user));
  else if (hipMalloc(reinterpret_cast<void**>(&d), (size_t)want) != hipSuccess) { (void)hipGetLastError(); d = nullptr; }
  if (!d) { set_error("device allocation of %llu bytes failed", (unsigned long long)want); return FI_ENOMEM_DEVICE; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(d, g->image, (size_t)copy_bytes, hipMemcpyHostToDevice, s);
  g->last_h2d_bytes = copy_bytes; g->last_h2d_copies = 1;
  if (e == hipSuccess && !g->gathered)
    for (const Member& mb : g->members) {
      e = hipMemcpyAsync(d + mb.arena_off, mb.spec.weights, (size_t)mb.plan.packed_bytes, hipMemcpyHostToDevice, s);
      if (e != hipSuccess) break;
      g->last_h2d_bytes += mb.plan.packed_bytes; ++g->last_h2d_copies;
    }
  if (e != hipSuccess) {
    set_error("hipMemcpyAsync: %s", hipGetErrorString(e));
    if (g->opts.dev_free) g->opts.dev_free(d, g->opts.user); else (void)hipFree(d);
    return FI_EHIP;
  }
  if (!g->copy_done && hipEventCreateWithFlags(&g->copy_done, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); g->copy_done = nullptr; }
  if (g->copy_done) { (void)hipEventRecord(g->copy_done, s); g->copy_pending.store(true); }
  else (void)hipStreamSynchronize(s);   // no event to order later runs after the copy: finish it here
  ensure_lanes(g);
  g->dev = d;
  g->dev_capacity = want;
  g->state = 1;
  ++g->n_loads;
  return FI_OK;
}

// The weight copy of a load or a member swap is asynchronous on the stream it was given.  A pass may be issued
// to any other stream (a lane worker's, a caller's second stream), so every pass first orders its stream after
// that copy; once the copy is known to have finished the wait is skipped.
static void order_after_copy(fi_dag* g, hipStream_t s) {
  if (!g->copy_done || !g->copy_pending.load(std::memory_order_acquire)) return;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cs) != hipSuccess) (void)hipGetLastError();
  if (cs != hipStreamCaptureStatusNone) return;   // a caller recording this stream has ordered it after the load itself
  if (hipEventQuery(g->copy_done) == hipSuccess) { g->copy_pending.store(false, std::memory_order_release); return; }
  (void)hipGetLastError();   // hipErrorNotReady is not an error here
  (void)hipStreamWaitEvent(s, g->copy_done, 0);
}

// ms: durations with every launch serialised on the caller's stream.  tl_begin / tl_end: the schedule as
// fi_run issues it (lanes concurrent), launch i spanning [previous event on its stream, event after it],
// in milliseconds since the pass began.
static fi_status run_impl(fi_dag* g, const void* d_input, int32_t batch, void* const* d_outputs, void* stream,
                          float* ms, int32_t n_ms, float* tl_begin = nullptr, float* tl_end = nullptr,
                          const void* const* d_inputs = nullptr, const int32_t* batches = nullptr, int32_t only_lane = -1,
                          uint8_t* workspace = nullptr) {
  if (!g || (!d_input && !d_inputs) || !d_outputs) { set_error("null argument"); return FI_EINVAL; }
  if (d_inputs && !g->opts.per_member_inputs) { set_error("per-member inputs need a DAG built with per_member_inputs"); return FI_ESTATE; }
  if (g->state != 1) { set_error("fi_run: handle is not loaded"); return FI_ESTATE; }
  if (only_lane >= g->n_lanes) { set_error("lane %d outside [0, %d)", only_lane, g->n_lanes); return FI_EINVAL; }
  if (!batches && (batch < 1 || batch > g->opts.max_batch)) { set_error("batch %d outside [1, %d]", batch, g->opts.max_batch); return FI_EINVAL; }
  // members that take part in this pass: those of the lane asked for (all lanes by default) that bring an image
  auto idle = [&](size_t m) { return (only_lane >= 0 && g->members[m].lane != only_lane) || (batches && batches[m] == 0); };
  for (size_t m = 0; m < g->members.size(); ++m) {
    if (idle(m)) continue;
    if (batches && (batches[m] < 0 || batches[m] > g->opts.max_batch)) { set_error("batch %d of member %zu outside [0, %d]", batches[m], m, g->opts.max_batch); return FI_EINVAL; }
    if (d_inputs && !d_inputs[m]) { set_error("input %zu is null", m); return FI_EINVAL; }
    if (!d_outputs[m]) { set_error("output %zu is null", m); return FI_EINVAL; }
  }
  const size_t nl = g->launches.size();
  const bool timeline = tl_begin && tl_end;
  if ((ms || timeline) && n_ms < (int32_t)nl) { set_error("timing arrays hold %d entries, schedule has %zu launches", n_ms, nl); return FI_EINVAL; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!g->capturing) order_after_copy(g, s);
  std::vector<hipEvent_t> ev;
  std::vector<size_t> ev_before;                               // timeline: index of the event that precedes launch i on its stream
  std::vector<size_t> last_on_lane;
  if (ms || timeline) {
    ev_before.assign(nl, 0);
    last_on_lane.assign((size_t)g->n_lanes, 0);
    ev.resize(nl + 1);
    for (auto& e : ev) if (hipEventCreate(&e) != hipSuccess) { set_error("hipEventCreate failed"); return FI_EHIP; }
    (void)hipEventRecord(ev[0], s);
  }
  KArgs a{};
  a.wbase = g->dev;
  a.abase = g->dev + g->arena_bytes;
  a.wsbase = workspace ? workspace : a.abase + g->act_bytes;   // the workspace follows the activation arena
  fi_status rc = FI_OK;
  // Lanes: after the shared input is staged on the caller's stream the internal streams fork from
  // it, every launch goes to its lane's stream, and the caller's stream joins them at the end.
  const bool lanes = !ms && !g->opts.use_graph && g->n_lanes > 1 && only_lane < 0 &&
                     (int32_t)g->lane_streams.size() >= g->n_lanes - 1 && (int32_t)g->lane_events.size() >= g->n_lanes;
  bool forked = false;
  for (size_t i = 0; i < nl; ++i) {
    const Launch& L = g->launches[i];
    if (only_lane >= 0 && L.kind != K_STAGE && L.lane != only_lane) continue;   // another lane's launch
    if (lanes && !forked && L.level > 0) {
      (void)hipEventRecord(g->lane_events[0], s);
      for (int32_t l = 1; l < g->n_lanes; ++l) (void)hipStreamWaitEvent(g->lane_streams[(size_t)l - 1], g->lane_events[0], 0);
      forked = true;
    }
    hipStream_t ls = (lanes && L.lane > 0) ? g->lane_streams[(size_t)L.lane - 1] : s;
    a.n = L.n;
    for (int32_t k = 0; k < L.n && L.kind == K_STAGE; ++k) {
      const StageTensor& st = g->stages[(size_t)L.nodes[(size_t)k]];
      a.ext_in[k] = (d_inputs && st.member >= 0) ? d_inputs[st.member] : d_input;
      a.batch[k] = (batches && st.member >= 0) ? batches[st.member] : batch;
      if (st.member >= 0 && idle((size_t)st.member)) a.batch[k] = 0;   // staged by its own lane's pass
    }
    for (int32_t k = 0; k < L.n && L.kind != K_STAGE; ++k) {
      const Node& nd = g->nodes[(size_t)L.nodes[(size_t)k]];
      a.ext_out[k] = nd.is_output ? d_outputs[nd.model] : nullptr;
      a.batch[k] = idle((size_t)nd.model) ? 0 : batches ? batches[nd.model] : batch;   // a member with no image this pass gets no workgroup
    }
    const int e = launch_kernel(L, a, ls, g->descs);
    if (e != (int)hipSuccess) { set_error("launch %zu (%s): %s", i, L.name.c_str(), hipGetErrorString((hipError_t)e)); rc = FI_EHIP; break; }
    if (ms) (void)hipEventRecord(ev[i + 1], s);
    if (timeline) {
      const size_t lane = lanes ? (size_t)L.lane : 0;
      // before the fork every lane's history is the caller's stream
      ev_before[i] = (lanes && !forked) ? last_on_lane[0] : last_on_lane[lane];
      (void)hipEventRecord(ev[i + 1], ls);
      if (lanes && !forked) std::fill(last_on_lane.begin(), last_on_lane.end(), i + 1);
      else last_on_lane[lane] = i + 1;
    }
  }
  if (forked)
    for (int32_t l = 1; l < g->n_lanes; ++l) {
      (void)hipEventRecord(g->lane_events[(size_t)l], g->lane_streams[(size_t)l - 1]);
      (void)hipStreamWaitEvent(s, g->lane_events[(size_t)l], 0);
    }
  if (ms || timeline) {
    (void)hipStreamSynchronize(s);
    if (rc == FI_OK && ms)
      for (size_t i = 0; i < nl; ++i) (void)hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]);
    if (rc == FI_OK && timeline)
      for (size_t i = 0; i < nl; ++i) {
        tl_begin[i] = 0.0f;
        if (ev_before[i]) (void)hipEventElapsedTime(&tl_begin[i], ev[0], ev[ev_before[i]]);
        (void)hipEventElapsedTime(&tl_end[i], ev[0], ev[i + 1]);
      }
    for (auto& e : ev) (void)hipEventDestroy(e);
  }
  return rc;
}

static void drop_graph(fi_dag* g) {
  if (g->gexec) { (void)hipGraphExecDestroy(g->gexec); g->gexec = nullptr; }
}

fi_status fi_run(fi_dag* g, const void* d_input, int32_t batch, void* const* d_outputs, void* stream) {
  if (!g || !g->opts.use_graph || !stream) return run_impl(g, d_input, batch, d_outputs, stream, nullptr, 0);
  // One HIP graph holds the whole schedule; it is rebuilt when the batch or a buffer changes.
  if (!d_input || !d_outputs) { set_error("null argument"); return FI_EINVAL; }
  if (g->state != 1) { set_error("fi_run: handle is not loaded"); return FI_ESTATE; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool same = g->gexec && g->g_batch == batch && g->g_input == d_input;
  for (size_t m = 0; same && m < g->members.size(); ++m) same = g->g_outputs[m] == d_outputs[m];
  order_after_copy(g, s);
  if (!same) {
    drop_graph(g);
    hipGraph_t graph = nullptr;
    if (hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) != hipSuccess) {
      (void)hipGetLastError();
      return run_impl(g, d_input, batch, d_outputs, stream, nullptr, 0);  // this stream cannot capture
    }
    g->capturing = true;
    const fi_status rc = run_impl(g, d_input, batch, d_outputs, stream, nullptr, 0);
    g->capturing = false;
    const hipError_t e = hipStreamEndCapture(s, &graph);
    if (rc != FI_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess || !graph) { set_error("hipStreamEndCapture: %s", hipGetErrorString(e)); return FI_EHIP; }
    const hipError_t ei = hipGraphInstantiate(&g->gexec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (ei != hipSuccess) { g->gexec = nullptr; set_error("hipGraphInstantiate: %s", hipGetErrorString(ei)); return FI_EHIP; }
    g->g_batch = batch;
    g->g_input = d_input;
    g->g_outputs.assign(d_outputs, d_outputs + g->members.size());
  }
  const hipError_t e = hipGraphLaunch(g->gexec, s);
  if (e != hipSuccess) { set_error("hipGraphLaunch: %s", hipGetErrorString(e)); return FI_EHIP; }
  return FI_OK;
}

fi_status fi_run_static(fi_dag* g, const void* d_input, int32_t batch, void* const* d_outputs, void* stream) {
  if (!g) { set_error("null handle"); return FI_EINVAL; }
  if (g->workspace_bytes > FI_STATIC_SCRATCH_BYTES) {
    set_error("fi_run_static: the DAG's split-K workspace is %llu bytes, the static array holds %llu (use fi_run)",
              (unsigned long long)g->workspace_bytes, (unsigned long long)FI_STATIC_SCRATCH_BYTES);
    return FI_EBUDGET;
  }
  void* ws = nullptr;
  uint64_t ws_bytes = 0;
  const int e = static_scratch(&ws, &ws_bytes);
  if (e != (int)hipSuccess || !ws || ws_bytes < g->workspace_bytes) {
    set_error("fi_run_static: no static workspace on this device: %s", hipGetErrorString((hipError_t)e));
    return FI_EHIP;
  }
  // Partial sums are written in full by the split launch before the reduce launch reads them: nothing in the array
  // has to start at zero, whatever an earlier call left there.
  return run_impl(g, d_input, batch, d_outputs, stream, nullptr, 0, nullptr, nullptr, nullptr, nullptr, -1, static_cast<uint8_t*>(ws));
}

fi_status fi_run_inputs(fi_dag* g, const void* const* d_inputs, int32_t batch, void* const* d_outputs, void* stream) {
  if (!d_inputs) { set_error("null inputs"); return FI_EINVAL; }
  return run_impl(g, nullptr, batch, d_outputs, stream, nullptr, 0, nullptr, nullptr, d_inputs);
}

fi_status fi_run_batches(fi_dag* g, const void* const* d_inputs, const int32_t* batches, void* const* d_outputs, void* stream) {
  if (!d_inputs || !batches) { set_error("null inputs or batches"); return FI_EINVAL; }
  return run_impl(g, nullptr, 0, d_outputs, stream, nullptr, 0, nullptr, nullptr, d_inputs, batches);
}

fi_status fi_run_lane(fi_dag* g, int32_t lane, const void* const* d_inputs, const int32_t* batches, void* const* d_outputs, void* stream) {
  if (!d_inputs || !batches) { set_error("null inputs or batches"); return FI_EINVAL; }
  if (lane < 0) { set_error("lane %d is negative", lane); return FI_EINVAL; }
  return run_impl(g, nullptr, 0, d_outputs, stream, nullptr, 0, nullptr, nullptr, d_inputs, batches, lane);
}

fi_status fi_profile(fi_dag* g, const void* d_input, int32_t batch, void* const* d_outputs, void* stream, float* ms, int32_t n_ms) {
  if (!ms) { set_error("null ms"); return FI_EINVAL; }
  return run_impl(g, d_input, batch, d_outputs, stream, ms, n_ms);
}

fi_status fi_timeline(fi_dag* g, const void* d_input, int32_t batch, void* const* d_outputs, void* stream,
                      float* begin_ms, float* end_ms, int32_t n) {
  if (!begin_ms || !end_ms) { set_error("null timeline array"); return FI_EINVAL; }
  return run_impl(g, d_input, batch, d_outputs, stream, nullptr, n, begin_ms, end_ms);
}

fi_status fi_swap_model(fi_dag* g, int32_t slot, const fi_model_spec* model, void* stream) {
  if (!g || !model) { set_error("null argument"); return FI_EINVAL; }
  if (slot < 0 || slot >= (int32_t)g->members.size()) { set_error("slot %d outside [0, %zu)", slot, g->members.size()); return FI_EINVAL; }
  // Plan on a scratch handle: a failure leaves the DAG as it was.  The other members keep their
  // arena offsets (their weights stay where they are); the newcomer takes the lowest gap that holds it.
  fi_dag t;
  t.opts = g->opts;
  t.members = g->members;
  Member& nm = t.members[(size_t)slot];
  nm = Member{};
  nm.spec = *model;
  const fi_model_spec* first = g->members.size() > 1 ? &g->members[slot == 0 ? 1 : 0].spec : nullptr;
  fi_status st = analyze_member(t.opts, nm, slot, first);
  if (st != FI_OK) return st;
  st = plan_dag(&t);
  if (st != FI_OK) return st;
  if (g->state == 1 && t.device_bytes > g->dev_capacity) {
    set_error("after the swap the DAG needs %llu device bytes, the loaded allocation holds %llu (unload and rebuild, or load with more swap_headroom_bytes)",
              (unsigned long long)t.device_bytes, (unsigned long long)g->dev_capacity);
    return FI_EBUDGET;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Member& placed = t.members[(size_t)slot];
  const uint8_t* src = static_cast<const uint8_t*>(placed.spec.weights);
  if (!g->gathered && g->image && !placed.spec.weights_packed) {   // a canonical newcomer has to be packed somewhere: from now on the handle keeps an image
    if (g->opts.load_mode != FI_LOAD_AUTO || !gather_image(g)) { set_error("a member in canonical layout needs the handle's pinned image"); return FI_ENOMEM_HOST; }
  }
  const bool one_copy = g->gathered && g->image;
  if (one_copy) {
    // the pinned image stays the exact image of the arena; copies out of it must have finished
    if (g->copy_done) (void)hipEventSynchronize(g->copy_done);
    if (t.arena_bytes > g->image_capacity) {
      uint8_t* bigger = static_cast<uint8_t*>(pin_alloc(g->opts, (size_t)t.arena_bytes));
      if (!bigger) { set_error("pinned allocation of %llu bytes failed", (unsigned long long)t.arena_bytes); return FI_ENOMEM_HOST; }
      parallel_copy(bigger, g->image, std::min(g->image_bytes, g->image_capacity));   // same contents, more room: the DAG is unchanged
      pin_free(g->opts, g->image);
      g->image = bigger;
      g->image_capacity = t.arena_bytes;
    }
    if (placed.spec.weights_packed) parallel_copy(g->image + placed.arena_off, src, placed.plan.packed_bytes);
    else pack_model(placed.spec, placed.plan, g->image + placed.arena_off);
    src = g->image + placed.arena_off;
  }
  if (g->state == 1) {
    const hipError_t e = hipMemcpyAsync(g->dev + placed.arena_off, src, (size_t)placed.plan.packed_bytes, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) {
      set_error("hipMemcpyAsync: %s", hipGetErrorString(e));
      if (one_copy) {   // the DAG stays as it was, so its image must too: the outgoing member goes back where the newcomer was written
        const Member& old = g->members[(size_t)slot];
        if (old.spec.weights_packed) parallel_copy(g->image + old.arena_off, static_cast<const uint8_t*>(old.spec.weights), old.plan.packed_bytes);
        else pack_model(old.spec, old.plan, g->image + old.arena_off);
      }
      return FI_EHIP;
    }
    if (g->copy_done) { (void)hipEventRecord(g->copy_done, s); g->copy_pending.store(true); }
    else (void)hipStreamSynchronize(s);
    g->last_h2d_bytes = placed.plan.packed_bytes; g->last_h2d_copies = 1;
  }
  if (one_copy) g->image_bytes = t.arena_bytes;   // what the next load copies
  drop_graph(g);
  g->members = std::move(t.members);
  g->nodes = std::move(t.nodes);
  g->launches = std::move(t.launches);
  g->descs = std::move(t.descs);
  g->n_levels = t.n_levels; g->n_runs = t.n_runs; g->wdtype = t.wdtype; g->macs = t.macs; g->n_lanes = t.n_lanes;
  g->desc_bytes = t.desc_bytes; g->arena_bytes = t.arena_bytes; g->act_bytes = t.act_bytes;
  g->workspace_bytes = t.workspace_bytes; g->device_bytes = t.device_bytes;
  g->stages = std::move(t.stages);
  if (g->state == 1) ensure_lanes(g);
  return FI_OK;
}

fi_status fi_unload(fi_dag* g) {
  if (!g) { set_error("null handle"); return FI_EINVAL; }
  if (g->state != 1) { set_error("fi_unload: handle is not loaded"); return FI_ESTATE; }
  (void)hipDeviceSynchronize();
  drop_graph(g);
  for (hipStream_t ls : g->lane_streams) (void)hipStreamDestroy(ls);
  for (hipEvent_t ev : g->lane_events) (void)hipEventDestroy(ev);
  g->lane_streams.clear();
  g->lane_events.clear();
  if (g->copy_done) { (void)hipEventDestroy(g->copy_done); g->copy_done = nullptr; }
  if (g->opts.dev_free) g->opts.dev_free(g->dev, g->opts.user); else (void)hipFree(g->dev);
  g->dev = nullptr;
  g->dev_capacity = 0;
  g->state = 0;
  return FI_OK;
}

void fi_destroy(fi_dag* g) {
  if (!g) return;
  if (g->state == 1) (void)fi_unload(g);
  pin_free(g->opts, g->image);
  delete g;
}

}  // extern "C"

namespace fi {
void serving_info(const fi_dag* g, ServingInfo* out) {
  out->n_models = (int32_t)g->members.size();
  out->max_batch = g->opts.max_batch;
  out->per_member_inputs = g->opts.per_member_inputs;
  out->state = g->state;
  const fi_model_spec& m0 = g->members[0].spec;
  out->image_bytes = (uint64_t)m0.in_h * m0.in_w * m0.in_c * esize(m0.dtype);
  out->out_bytes.assign(g->members.size(), 0);
  for (const Node& nd : g->nodes)
    if (nd.is_output) out->out_bytes[(size_t)nd.model] = (uint64_t)nd.Ho * nd.Wo * nd.Co * 4;
  out->lane.clear();
  for (const Member& mb : g->members) out->lane.push_back(mb.lane);
  out->n_lanes = g->n_lanes;
  out->opts = g->opts;
}
}  // namespace fi
