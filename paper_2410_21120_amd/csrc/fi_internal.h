// Internal structures shared by the host planner, the packer and the kernels.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/fusedinf.h"

namespace fi {

constexpr uint64_t kAlign = 256;       // every arena object starts on a 256-byte boundary
constexpr uint64_t kNone = ~0ull;
// Largest sizes a spec may name.  They keep the planner's and the kernels' 32-bit index arithmetic exact:
// rows of an implicit GEMM (batch x pixels) and elements of one tensor per image stay below 2^31.
constexpr int32_t kMaxChannels = 1 << 18;   // channels of any tensor
constexpr int32_t kMaxSide = 1 << 14;       // input height / width
constexpr int32_t kMaxWindow = 1 << 10;     // kernel size, stride, padding as spec fields (kernels themselves stop at 15)
constexpr int32_t kMaxElems = 1 << 28;      // elements of one tensor, per image (padded channels included)
constexpr int32_t kMaxBatch = 1 << 16;
inline uint64_t align_up(uint64_t v, uint64_t a = kAlign) { return (v + a - 1) / a * a; }

// Kernel families.  A launch runs one family over 1..FI_MAX_GROUP problems.
enum Kind : int32_t {
  K_STAGE = 0,        // caller's NHWC input -> channel-padded copy in the activation arena
  K_CONV_DIRECT = 1,  // one thread per output element (fp32 models, fp32-activation members)
  K_CONV_MFMA = 2,    // implicit GEMM on the matrix cores (bf16 weights, bf16 activations)
  K_DWCONV = 3,
  K_MAXPOOL = 4,
  K_GAP = 5,
  K_SOFTMAX = 6,
  K_FC = 7,           // small-batch fully connected: weight-streaming split-K partial products
  K_REDUCE = 8,       // finishes a split-K node: sums partials, bias, residual, activation, store
  K_CONCAT = 9,       // channels of the first source, then of the second
  K_AVGPOOL = 10,     // window average (divisor k*k)
  K_MUL = 11,         // per-(image, channel) gate
  K_GATHER = 12,      // channel slice (stride == 0: channels from pad on) or shuffle (stride == 1: k groups)
  K_CHAIN = 13,       // a convolution and the one or two pointwise convolutions behind it, per 128-pixel tile, in one launch
  K_STEM = 14,        // a 7x7 stride-2, 3x3 stride-1 or 3x3 stride-2 convolution over the 4-channel model input, from an input patch
                      // in LDS (tile bit 0 clear), or a stride-2 one and the 3x3 stride-2 max-pool that alone reads it (tile bit 0
                      // set: the pool node carries the launch); tile bits 1.. = which convolution
  K_NKINDS
};

// Tile shapes of the MFMA implicit GEMM (rows = output pixels, cols = output channels).
// T_128x128_DEEP: the 128x128 tile with three reduction tiles in flight in registers instead of one (long reductions in
// launches of few workgroups).
enum Tile : int32_t { T_128x128 = 0, T_128x64 = 1, T_64x64 = 2, T_256x128 = 3, T_256x64 = 4, T_128x128_DEEP = 5, T_NTILES };
#ifdef __HIPCC__
#define FI_HD __host__ __device__
#else
#define FI_HD
#endif
FI_HD inline int tile_bm(int t) { return (t == T_256x128 || t == T_256x64) ? 256 : t == T_64x64 ? 64 : 128; }
FI_HD inline int tile_bn(int t) { return (t == T_128x128 || t == T_256x128 || t == T_128x128_DEEP) ? 128 : 64; }

// Problem descriptor: one node of the fused DAG, batch independent, handed to the kernels
// as launch arguments.  Tensor offsets are relative to the activation region, weight offsets
// to the weight arena.
struct Desc {
  uint64_t x_off, y_off, r_off;  // input / output / second operand: residual, gate, second source of a concatenation or of an
                                 // interleaving shuffle (kNone = none)
  uint64_t w_off, b_off;
  int32_t H, W, C, Cp;           // input: logical dims and padded channel stride
  int32_t Ho, Wo, Co, Cop;       // output
  int32_t k, stride, pad, act;   // channel gather: k = shuffle groups, pad = first channel of a slice, stride = mode
                                 // (0 slice, 1 shuffle, 2 interleave two sources)
  int32_t Kp;                    // padded reduction length of a weight row (elements); concatenation: channels of the second source
  int32_t ext;                   // 1: output is the caller's fp32 buffer of this problem
  int32_t out_f32;               // 1: output stored as fp32 whatever the activation dtype
  int32_t tiles_n;               // MFMA conv: column tiles; FC: 32-feature tiles; depthwise / pooling strip kernels: outputs per
                                 // thread along a row; concatenation / interleaving shuffle: pixel stride of the second source;
                                 // stem launch: workgroups that share the problem
  int32_t vec;                   // 1: bf16 tensors with Cp % 8 == 0, kernels work on 8-channel vectors
  int32_t splits;                // reduction splits (>1: fp32 partials [splits][rows][Cop] at ws_off)
  uint64_t ws_off;               // split-K partials, relative to the workspace base (KArgs::wsbase)
  int32_t kw, pad_w;             // dense conv: kernel width and horizontal padding (k, pad are the vertical ones)
  int32_t gin, gout;             // MFMA conv of a grouped convolution: input / output channels per group (0 = dense walk over all channels);
                                 // stem launch: height / width of the convolution's output (Ho, Wo are the stored tensor's: the pooled size
                                 // when the pool is part of the launch)
  int32_t xs, ys;                // elements between neighbouring pixels of the input / output: Cp / Cop, or the channel stride of the
                                 // concatenation the tensor is stored inside (read by the depthwise kernels and by MFMA convolutions
                                 // with an input-side stage, written by the bf16 vector kernels and the MFMA convolution; every other
                                 // kernel sees xs == Cp, ys == Cop: launch_kernel checks)
  uint64_t pw_off, pb_off;       // MFMA conv with a stage on its input side.  pre_kind 1, per-channel affine: scale (bf16 [Cp]) and
                                 // shift (fp32 [Cp]) in the weight arena.  pre_kind 2, per-(image, channel) gate: pw_off is the gate
                                 // tensor [batch][Cp] (bf16) in the activation region.  kNone where unused
  int32_t pre_act, pre_kind;     // activation of the affine stage; 0 = no stage.  Stem launch with the pool: pre_act is the pool's padding
};
static_assert(sizeof(Desc) == 168, "Desc is 168 bytes");

struct Node {
  int32_t model, index;
  int32_t op, act;
  int32_t input, residual;       // global node ids (or -1 / -2)
  int32_t H, W, C, Cp, Ho, Wo, Co, Cop, k, stride, pad;
  int32_t kw, pad_w;             // dense conv: kernel width / horizontal padding (k / pad are the vertical ones)
  int32_t Kp;
  int32_t groups;                // conv2d: channel groups (1 = dense)
  int32_t root, chan;            // root >= 0: the tensor is stored inside concatenation node `root`, from channel `chan` on, with
                                 // that node's channel stride, and has no buffer of its own
  int32_t elided;                // no launch: a concatenation whose sources are both stored in place, a per-channel affine or
                                 // scaling node that the convolution reading it applies while loading its input, or (2) a
                                 // concatenation that the two-group shuffle reading it replaces by interleaving its sources
  int32_t pre;                   // MFMA conv: the node fused into its input side, a per-channel affine (depthwise 1x1) or a
                                 // squeeze-excite scaling; shuffle: the concatenation it replaces; max-pool run by a stem launch: the
                                 // convolution in front of it (-1 = none)
  int32_t chain, chain_pos;      // chain >= 0: the node runs inside the chained launch headed by node `chain`, as its first (0), second
                                 // (1) or third (2) convolution; the head's own output is stored nowhere
  int32_t level;                 // depth: 1 + the deepest input
  int32_t run;                   // position in the launch order (launches are issued by ascending `run`): the depth, unless the node
                                 // follows a chain's head (then the head's) or its member's early levels are run in member chunks
  int32_t out_dtype;             // FI_F32 / FI_BF16 as stored
  int32_t is_output;
  int32_t first_level, last_level;
  int32_t launch, slot;          // launch index and problem slot inside it
  int32_t lane;                  // lane of the node's member
  int32_t kind, tile;
  int32_t splits;                // reduction splits (1 = none)
  uint64_t ws_off;               // partials of a split node, relative to the workspace
  uint64_t w_rel, b_rel;         // offsets inside the member's packed blob
  uint64_t w_off, b_off;         // offsets in the weight arena
  uint64_t out_off, out_bytes;   // activation arena placement (bytes at max_batch)
  uint64_t macs;
};

struct Launch {
  int32_t level, kind, tile;
  int32_t lane;                  // stream the launch is issued to (0 = the caller's)
  int32_t wdtype, adtype;        // weight / activation storage dtype of every problem in it
  int32_t first_desc, n;         // contiguous range in the descriptor table
  std::vector<int32_t> nodes;    // global node ids, slot order
  std::string name;
  uint64_t macs, act_bytes, weight_bytes;
};

// Per-member analysis shared by fi_model_packed_size / fi_model_pack / fi_build_dag.
struct ModelPlan {
  std::vector<Node> nodes;       // input/residual are LOCAL indices here
  uint64_t packed_bytes = 0;
  int32_t cgran = 1;             // channel padding granule (8 for bf16 weights, 1 for fp32)
  int32_t in_cp = 0;
};

// Arguments every kernel receives by value.
struct KArgs {
  const uint8_t* wbase;          // weight arena (device)
  uint8_t* abase;                // activation region (device)
  uint8_t* wsbase;               // split-K workspace (device): the tail of the loaded allocation, or the library's static array
  int32_t n, reserved;
  int32_t batch[FI_MAX_GROUP];   // images per problem slot in this pass (members may bring batches of their own)
  int32_t first_block[FI_MAX_GROUP + 1];  // workgroup index where each problem starts (filled per launch)
  const void* ext_in[FI_MAX_GROUP];  // caller's input per problem slot (K_STAGE only)
  void* ext_out[FI_MAX_GROUP];   // caller's output per problem slot (when Desc.ext)
  Desc d[FI_MAX_GROUP];          // the launch's problems: read through the scalar cache, no memory round trip
};

// What the request aggregator needs to know about a handle (filled by serving_info in fi_api.cpp).
struct ServingInfo {
  int32_t n_models = 0, max_batch = 0, per_member_inputs = 0, state = 0;
  uint64_t image_bytes = 0;                 // one input image [in_h, in_w, in_c] in the weight dtype
  std::vector<uint64_t> out_bytes;          // one output row of every member (fp32)
  std::vector<int32_t> lane;                // launch lane of every member
  int32_t n_lanes = 1;
  fi_build_opts opts{};                     // allocator callbacks
};
void serving_info(const fi_dag* dag, ServingInfo* out);

// Copies n rows of `bytes` bytes each, row i from src[i] to dst[i] (device pointers, 16-byte aligned, bytes a
// multiple of 16), with as few kernel launches as the argument space allows (kCopyRows rows per launch): the
// request aggregator gathers and scatters a pass's images with it instead of issuing one copy per request.
constexpr int32_t kCopyRows = 64;
int launch_copy_rows(const void* const* src, void* const* dst, int32_t n, uint64_t bytes, void* stream);

void set_error(const char* fmt, ...);
fi_status analyze_model(const fi_model_spec& m, ModelPlan& out);
void pack_model(const fi_model_spec& m, const ModelPlan& p, uint8_t* dst);

// The library's static split-K workspace on the current device (fi_run_static): its device address and size.
// Implemented in fi_kernels.hip; returns a hipError_t as int.  Allocates nothing.
int static_scratch(void** ptr, uint64_t* bytes);

// Implemented in fi_chain.hip: a K_CHAIN launch (problems are triples of descriptors).  Returns a hipError_t as int.
int launch_chain(const Launch& L, const KArgs& a, void* stream, const std::vector<Desc>& host_descs);

// Implemented in fi_stem.hip: a K_STEM launch, and the workgroups one of its problems takes.  Returns a hipError_t as int.
int launch_stem(const Launch& L, const KArgs& a, void* stream, const std::vector<Desc>& host_descs);
int stem_blocks(int tile, const Desc& d, int batch);
// A stem launch's tile field: bit 0 = the pool is part of the launch, bits 1.. = the convolution's geometry
// (0: 7x7 stride 2, 1: 3x3 stride 1, 2: 3x3 stride 2; -1: none of them).
inline int stem_geometry(int k, int kw, int stride) {
  if (k != kw) return -1;
  if (k == 7 && stride == 2) return 0;
  if (k == 3 && stride == 1) return 1;
  if (k == 3 && stride == 2) return 2;
  return -1;
}

// Implemented in fi_kernels.hip.  Returns a hipError_t as int; `stream` is a hipStream_t.
int launch_kernel(const Launch& L, const KArgs& a, void* stream, const std::vector<Desc>& host_descs);

}  // namespace fi
