/* fusedinf.h -- C ABI of the fused multi-model CNN inference library (gfx950).
 *
 * The library implements the hot path of FusedInf (Section IV "System Design",
 * Algorithm 1): several independent CNN inference models are compiled into ONE
 * DAG -- the disjoint union of the members' layer graphs, no edge between members
 * -- which is then loaded, executed and swapped as a unit.  "Efficient memory
 * allocation" and "Fewer memory calls" (Section IV-B) become: one device
 * allocation per load, holding one contiguous weight arena for all members that
 * is filled by one pinned-host-to-device copy.  The inference loop of Algorithm 1
 * (every node evaluates phi(sum_j u_j x_j) on tensors of its own model) becomes
 * one launch schedule in which nodes of different members at the same depth run
 * as grouped kernels; members of different architecture, which rarely share a
 * kernel shape, form separate lanes of that schedule that run concurrently.
 * Properties C1 / C4 (Section III-A, Section IV-C) are kept: no operator is
 * merged across members, each member's output is bit-identical to the member run
 * alone, and no member reads another member's tensors.
 *
 * Conventions
 *  - Every call returns fi_status; on error out-parameters are untouched and
 *    fi_last_error() holds a thread-local message.  No exception crosses the ABI.
 *  - "host" / "device" is stated for every pointer.  Specs and host weight blobs
 *    are BORROWED: the caller keeps them alive until fi_destroy().
 *  - State machine:  BUILT --fi_load--> LOADED --fi_run*--> LOADED --fi_unload-->
 *    BUILT --fi_destroy--> gone.  Any other transition returns FI_ESTATE.
 *  - All members of one DAG share the weight dtype and the input shape.  fi_run
 *    feeds one shared input batch to every member; fi_run_inputs gives each
 *    member an input of its own (Algorithm 1's per-model inputs x^m).
 *  - Buffers: a run over `batch` images reads batch x fi_dag_info.input_image_bytes
 *    bytes from every input pointer it is given and writes batch x
 *    fi_member_info.output_row_bytes bytes to each member's output pointer.  The
 *    library cannot see how much memory stands behind a pointer: size the buffers
 *    from those two figures.
 *  - The planner may fold a node into its neighbours (a concatenation written in
 *    place by its producers, a per-channel affine or squeeze-excite scaling
 *    applied by the convolution that reads it, a concatenation that a shuffle
 *    interleaves): such a node has no launch and no tensor of its own, and every
 *    output keeps the bits of the unfolded schedule (fi_build_opts.copy_concats,
 *    fi_build_opts.separate_affine switch the folding off).
 */
#ifndef FUSEDINF_H
#define FUSEDINF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fi_dag fi_dag; /* opaque, owned by the library, one per fi_build_dag */

typedef enum {
  FI_OK = 0,
  FI_EINVAL = 1,        /* malformed spec / argument (cycle, dangling index, shape mismatch) */
  FI_EUNSUPPORTED = 2,  /* well-formed but outside what the kernels cover */
  FI_ESTATE = 3,        /* call not allowed in the handle's current state */
  FI_ENOMEM_HOST = 4,   /* host / pinned allocation failed */
  FI_ENOMEM_DEVICE = 5, /* device allocation failed; handle stays BUILT */
  FI_EBUDGET = 6,       /* DAG needs more device bytes than fi_build_opts.max_device_bytes */
  FI_EHIP = 7           /* a HIP runtime call failed */
} fi_status;

typedef enum { FI_F32 = 0, FI_BF16 = 1 } fi_dtype;
typedef enum { FI_CONV2D = 0, FI_DWCONV2D = 1, FI_MAXPOOL2D = 2, FI_GLOBAL_AVGPOOL = 3, FI_FC = 4, FI_SOFTMAX = 5, FI_CONCAT = 6, FI_AVGPOOL2D = 7, FI_MUL = 8, FI_SLICE = 9, FI_SHUFFLE = 10 } fi_op;
/* hard sigmoid h(v) = min(max(v + 3, 0), 6) / 6, hard swish v * h(v); sigmoid s(v) = 1 / (1 + exp(-v)), SiLU v * s(v) */
typedef enum { FI_ACT_NONE = 0, FI_ACT_RELU = 1, FI_ACT_RELU6 = 2, FI_ACT_HARDSWISH = 3, FI_ACT_HARDSIGMOID = 4,
               FI_ACT_SILU = 5, FI_ACT_SIGMOID = 6 } fi_act;

#define FI_INPUT (-1)       /* fi_layer_spec.input: the model's input tensor */
#define FI_NO_RESIDUAL (-2) /* fi_layer_spec.residual: nothing is added */
#define FI_MAX_GROUP 16     /* most problems one grouped launch carries */

/* One node u_i of a member's layer graph (Algorithm 1: node, its in-edge, its
 * activation phi_i).  Nodes are listed in topological order.
 *   conv2d / depthwise: y = act(conv(x, w) + b [+ residual]); cross-correlation,
 *     zero padding, floor output size.  Kernels are square (kh == kw) except that a
 *     dense conv2d may be rectangular (e.g. 1x7, 7x1); `pad` then applies only along the
 *     dimensions the kernel extends over (size > 1).  The residual
 *     is added BEFORE the activation.  Depthwise: cin == cout, one filter/channel.
 *     conv2d with groups = G > 1: output channel o sees only the input channels of
 *     its group o / (cout/G); canonical weights are then [cout][cin/G][kh][kw].  (Packed
 *     as block-diagonal dense rows: exact, at dense cost.)
 *   maxpool2d: max over in-range taps (padding acts as -inf); floor output size, or with
 *     ceil_mode the size rounded up (windows may hang over the far edge, the last one still
 *     starts inside the input or its leading padding).
 *   avgpool2d: in-range taps summed, divided by the window area kh*kw (zero padding counts),
 *     floor output size, one rounding on store.
 *   mul: `input` scaled per (image, channel) by the 1x1 tensor `residual` (the gate of a
 *     squeeze-and-excitation block); no activation.
 *   slice: channels [c_first, c_first + cout) of `input`.   shuffle: the channels, seen as a
 *     groups x (C/groups) matrix, transposed (output channel i*groups + g = input channel
 *     g*(C/groups) + i).  Both move values unchanged; no activation.
 *   concat: the channels of `input` followed by the channels of `residual` (here: the
 *     second source, same height and width); no activation.  cout = sum of both.
 *   global_avgpool: mean over H*W.   softmax: over the channel axis of a 1x1 tensor.
 *   fc: y = act(x W^T + b); cin = C*H*W of its input, flattened in (c,h,w) order.
 * w_off / b_off: byte offsets into the member's CANONICAL blob: weights
 * [cout][cin/groups][kh][kw] (fc: [cout][cin]) in the model dtype, bias [cout] fp32.
 * cin/cout of pooling, global_avgpool and softmax nodes are ignored (derived). */
typedef struct {
  int32_t op;       /* fi_op */
  int32_t input;    /* node index in this model, or FI_INPUT */
  int32_t residual; /* node index, or FI_NO_RESIDUAL */
  int32_t cin, cout, kh, kw, stride, pad;
  int32_t act;      /* fi_act */
  int32_t ceil_mode; /* maxpool2d only: 1 = output size rounds up */
  int32_t groups;    /* conv2d: channel groups (0 or 1 = dense), must divide cin and cout; shuffle: groups */
  int32_t c_first;   /* slice only: first channel taken */
  int32_t reserved;
  uint64_t w_off, b_off;
} fi_layer_spec;

/* One member model m.  `weights` (host) is either the canonical blob described
 * above (weights_packed == 0; the library converts it while building) or a blob
 * already in device layout written by fi_model_pack (weights_packed == 1; the
 * repository-time form that makes loading a pure copy).
 * act_dtype: storage precision of this member's intermediate tensors.  FI_BF16
 * (bf16 weights only) rounds every stored activation to bf16 once per node;
 * FI_F32 keeps activations in fp32 (mandatory for an FI_F32 model; for a bf16
 * model it buys fp32-grade accuracy at twice the activation traffic). */
typedef struct {
  const char* name;             /* host, borrowed, may be NULL */
  int32_t dtype;                /* fi_dtype of the weights */
  int32_t act_dtype;            /* fi_dtype of stored activations */
  int32_t in_c, in_h, in_w;     /* logical input [batch, in_c, in_h, in_w] */
  int32_t n_layers;
  const fi_layer_spec* layers;  /* host, borrowed */
  int32_t output_node;          /* node whose value is the member's prediction */
  int32_t weights_packed;       /* 0 canonical, 1 device layout (fi_model_pack) */
  const void* weights;          /* host, borrowed until fi_destroy */
  uint64_t weight_bytes;
} fi_model_spec;

typedef enum {
  FI_LOAD_ONE_COPY = 0,  /* gather members into one pinned image at build; fi_load = 1 H2D copy */
  FI_LOAD_PER_MODEL = 1, /* no host gather; fi_load copies each member's packed blob (+1 for the schedule) */
  FI_LOAD_AUTO = 2       /* gather only when it pays: members that are all in device layout are copied one by one
                          * straight out of the repository's blobs by the FIRST load of the handle (a set of models
                          * that is loaded once, as when the subset changes with every request, never pays a host
                          * gather); a handle that is loaded AGAIN gathers its image then, once, and from there on
                          * every load is one copy.  With a canonical member the image has to be written at build
                          * anyway and the mode is FI_LOAD_ONE_COPY. */
} fi_load_mode;

/* Allocator callbacks let the caller's memory pool (e.g. a tensor library's
 * caching allocator) back the library's memory.  NULL = hipMalloc / hipHostMalloc.
 * A callback returning NULL is reported as FI_ENOMEM_DEVICE / FI_ENOMEM_HOST. */
typedef struct {
  int32_t max_batch;         /* largest batch fi_run will be given (>= 1) */
  int32_t group_levels;      /* 1: same-depth nodes of different members share launches; 0: one launch per node */
  int32_t load_mode;         /* fi_load_mode */
  int32_t use_graph;         /* 1: fi_run replays the schedule as one HIP graph (needs a non-NULL stream) */
  int32_t serial_lanes;      /* 0: members of different architecture run concurrently on internal streams; 1: one stream */
  int32_t per_member_inputs; /* 1: every member reads an input of its own (fi_run_inputs); 0: one shared input */
  uint64_t max_device_bytes; /* 0 = unlimited; else fi_build_dag fails with FI_EBUDGET beyond it */
  void* (*dev_alloc)(size_t bytes, void* user);
  void (*dev_free)(void* ptr, void* user);
  void* (*pin_alloc)(size_t bytes, void* user);
  void (*pin_free)(void* ptr, void* user);
  void* user;
  uint64_t swap_headroom_bytes; /* extra device bytes fi_load allocates beyond the plan, for later fi_swap_model calls */
  int32_t copy_concats;      /* 0: producers whose only other readers allow it write straight into the concatenation's
                              * tensor and the concatenation needs no launch; 1: every concatenation copies its sources.
                              * The outputs are the same bits either way. */
  int32_t separate_affine;   /* 0: a per-channel affine node (1x1 depthwise, e.g. a DenseNet layer's normalisation + ReLU) or a
                              * squeeze-excite scaling (FI_MUL) read only by a 1x1 convolution is applied by that convolution
                              * while it loads its input and needs no launch; 1: it runs as a launch of its own.  The outputs
                              * are the same bits either way. */
  int32_t separate_chains;   /* 0: a dense convolution whose only reader is a 1x1 convolution (and that one's 1x1 reader, if it has
                              * one) runs with it in ONE launch per 128-pixel tile: the first output stays in registers, the second
                              * is written once and not read back (a ResNet bottleneck: 3x3 -> 1x1 expand -> the next block's 1x1
                              * reduce); 1: every convolution is a launch of its own.  The outputs are the same bits either way. */
  int32_t member_chunks;     /* 0 / 1: every level runs all members of a lane together.  c >= 2: the early, activation-heavy levels
                              * of a lane's members (up to the depth after which a member's live activations stay below two thirds
                              * of their peak) run for one chunk of ceil(members / c) members after the other, the deeper levels for
                              * all members together as ever: the chunks' early tensors share memory, so the activation arena shrinks,
                              * at the price of more, smaller launches.  The outputs are the same bits either way. */
  int32_t separate_stem;     /* 0: a 7x7 stride-2, 3x3 stride-1 or 3x3 stride-2 convolution over the model input with 64 output channels
                              * (the first layer of the ResNet-style families, of VGG, of SqueezeNet 1.1) runs from an input patch held on
                              * chip, and a 3x3 stride-2 max-pool (padding 0 or 1) that alone reads a stride-2 one runs in the same launch
                              * (the convolution's output is stored nowhere); 1: the
                              * general convolution kernel and a pooling launch of its own.  The outputs are the same bits either way. */
  int32_t reserved0;
} fi_build_opts;

typedef struct {
  uint64_t arena_bytes;      /* weight arena: schedule tables + every member's packed weights */
  uint64_t act_bytes;        /* activation arena at max_batch (liveness-planned) */
  uint64_t workspace_bytes;  /* kernel scratch */
  uint64_t device_bytes;     /* the one allocation fi_load makes = sum of the three (aligned) */
  uint64_t macs_per_image;   /* multiply-accumulates of conv/depthwise/fc nodes, all members */
  int32_t n_models, n_nodes, n_levels, n_launches;
  int32_t n_device_allocs;   /* device allocations per fi_load (1) */
  int32_t n_h2d_copies;      /* host-to-device copies per fi_load (1 in FI_LOAD_ONE_COPY) */
  int32_t state;             /* 0 BUILT, 1 LOADED */
  int32_t n_lanes;           /* concurrent launch lanes (groups of members with identical architecture) */
  uint64_t device_capacity;  /* bytes of the loaded allocation (device_bytes at load + swap headroom); 0 when BUILT */
  uint64_t last_h2d_bytes;   /* bytes moved by the most recent fi_load or fi_swap_model */
  int32_t last_h2d_copies;   /* copies issued by the most recent fi_load or fi_swap_model */
  int32_t reserved;
  uint64_t input_image_bytes; /* one input image [in_h, in_w, in_c] in the weight dtype: a run over `batch` images reads
                               * batch x this many bytes from the input pointer it is given, so size the buffer from it */
} fi_dag_info;

typedef struct {
  uint64_t arena_off, packed_bytes; /* placement of the member's packed weights in the weight arena */
  int32_t lane;                     /* launch lane of the member */
  int32_t first_node, n_nodes;      /* its nodes are [first_node, first_node + n_nodes) */
  int32_t reserved;
  uint64_t output_row_bytes;        /* one image's output row (fp32): a run writes batch x this many bytes to the member's output pointer */
} fi_member_info;

/* Introspection of the compiled DAG (tests, reports). */
typedef struct {
  int32_t model, index;      /* member and node index inside the member */
  int32_t op, level, launch; /* depth level (1-based) and the launch that executes it */
  int32_t out_c, out_h, out_w, out_cp; /* logical shape and padded channel stride of the output */
  int32_t out_dtype;         /* fi_dtype of the stored output */
  int32_t is_output;         /* 1: written to the caller's output buffer, not the arena */
  int32_t first_level, last_level; /* live range of the output tensor in levels */
  uint64_t out_off, out_bytes;     /* placement in the activation arena (at max_batch) */
  uint64_t w_off, b_off;           /* placement in the weight arena */
  uint64_t macs;                   /* per image */
} fi_node_info;

typedef struct {
  int32_t level, kind, n_problems, first_node; /* kind: internal kernel family id */
  int32_t lane, reserved;    /* launch lane (stream) */
  uint64_t macs_per_image;   /* dense work of the launch */
  uint64_t bytes_per_image;  /* compulsory activation bytes (in + out + residual), per image */
  uint64_t weight_bytes;     /* weight + bias bytes read once per launch */
  char name[32];             /* kernel family name, e.g. "conv_mfma_128x128" */
} fi_launch_info;

/* Section IV, "DNN model repository": the repository keeps every model ready to
 * be served, with its memory requirement.  Here: the size and the content of a
 * member's device-layout blob, computed at repository time on the host (no device
 * is touched).  model: host, borrowed for the call, canonical weights
 * (weights_packed == 0).  bytes: out, untouched on error.  FI_EINVAL for a null
 * argument or a malformed spec, FI_EUNSUPPORTED for an operator or size the
 * kernels do not cover. */
fi_status fi_model_packed_size(const fi_model_spec* model, uint64_t* bytes);
/* Same passage.  dst (host, caller-owned, ideally pinned) receives
 * fi_model_packed_size bytes: the exact image of the member's range in the weight
 * arena, so that a later load is a plain copy.  FI_EINVAL when dst_bytes is too
 * small or the blob is already packed; dst is then untouched. */
fi_status fi_model_pack(const fi_model_spec* model, void* dst, uint64_t dst_bytes);

/* Algorithm 1, DAG compilation: union the members' graphs, assign depth levels,
 * form grouped launches, lay out the weight arena and the activation arena.  Host
 * only: touches no device.  models: host array of n (1..) specs. */
fi_status fi_build_dag(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, fi_dag** out);
fi_status fi_query(const fi_dag* dag, fi_dag_info* info);
fi_status fi_node(const fi_dag* dag, int32_t i, fi_node_info* info);     /* i in [0, n_nodes) */
fi_status fi_launch(const fi_dag* dag, int32_t i, fi_launch_info* info); /* i in [0, n_launches) */
fi_status fi_member(const fi_dag* dag, int32_t m, fi_member_info* info); /* m in [0, n_models) */

/* The footprint fi_build_dag would report for these members (Section IV: the
 * repository knows every model's memory requirement, the manager sizes DAGs by
 * it), computed from the architectures alone: no pinned image is made and no
 * weight byte is read.  Same errors as fi_build_dag. */
fi_status fi_footprint(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, fi_dag_info* info);

/* Section IV-B, "Efficient memory allocation" and "Fewer memory calls": the whole
 * DAG gets ONE device allocation (weight arena, activation arena and workspace
 * together, through fi_build_opts.dev_alloc when given) and, in FI_LOAD_ONE_COPY,
 * ONE pinned-to-device copy of fi_dag_info.arena_bytes bytes (in
 * FI_LOAD_PER_MODEL: the 256-byte header plus one copy per member).  The copy is
 * asynchronous on hip_stream (a hipStream_t, NULL = default stream); every later
 * pass, on whichever stream it is issued, is ordered after it by the library.
 * BUILT -> LOADED.  FI_ESTATE when already loaded, FI_ENOMEM_DEVICE when the
 * allocation fails, FI_EHIP when a copy cannot be issued (the handle stays BUILT
 * and the allocation is returned). */
fi_status fi_load(fi_dag* dag, void* hip_stream);

/* Algorithm 1, DAG inference: one pass of the launch schedule, asynchronous on
 * hip_stream.  d_input: device, [batch, in_h, in_w, in_c] (NHWC) in the DAG's
 * weight dtype (fp32, or bf16 bit patterns), read-only, shared by all members.
 * d_outputs: HOST array of n_models DEVICE pointers; member m receives its output
 * node's value as fp32 [batch, out_h, out_w, out_c] (unpadded NHWC), i.e.
 * [batch, classes_m] logits for a classifier, or probabilities if the output
 * node is a softmax.  1 <= batch <= max_batch.  Allocates nothing. */
fi_status fi_run(fi_dag* dag, const void* d_input, int32_t batch, void* const* d_outputs, void* hip_stream);

/* For callers that cannot allocate device memory or let the library do it (code being
 * recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc): the
 * pass of fi_run, same arguments and same output bits, with the split-K partial sums
 * kept in a static device array of the library (FI_STATIC_SCRATCH_BYTES per GPU, held
 * until the process ends) instead of the workspace region of the loaded allocation.
 * Calls no hipMalloc / hipFree and no allocating library routine; always launches
 * eagerly (use_graph is ignored).  FI_EBUDGET when fi_dag_info.workspace_bytes exceeds
 * FI_STATIC_SCRATCH_BYTES (fi_run still serves such a DAG).  Every call on a GPU shares
 * that GPU's array: two calls that overlap in time on one GPU, from whichever handle,
 * stream or thread, race on it.  Nothing in the array needs clearing between calls. */
#define FI_STATIC_SCRATCH_BYTES (32u << 20)
fi_status fi_run_static(fi_dag* dag, const void* d_input, int32_t batch, void* const* d_outputs, void* hip_stream);

/* Algorithm 1 gives every member model m its own input x^m: the same pass with
 * d_inputs a HOST array of n_models DEVICE pointers, member m reading
 * d_inputs[m] ([batch, in_h, in_w, in_c] NHWC in the weight dtype, read-only; all
 * members share the input shape and the batch).  Needs a DAG built with
 * fi_build_opts.per_member_inputs = 1 (else FI_ESTATE); such a DAG stages one
 * channel-padded copy per member instead of one per activation dtype and channel
 * stride, and fi_run
 * on it feeds the one input to every member.  Always launches eagerly (use_graph
 * applies to fi_run). */
fi_status fi_run_inputs(fi_dag* dag, const void* const* d_inputs, int32_t batch, void* const* d_outputs, void* hip_stream);

/* The same pass when the members have gathered different numbers of requests
 * (Section IV: the manager aggregates, per model, the requests that arrived while
 * the device was busy): member m runs on batches[m] images (HOST array of n_models
 * entries, 0 <= batches[m] <= max_batch) read from d_inputs[m] and writes
 * [batches[m], classes_m] to d_outputs[m].  A member with batches[m] == 0 sits the
 * pass out: none of its kernels get a workgroup, its pointers may be NULL and its
 * output buffer is not touched.  An image's output bits do not depend on the batch
 * it travels in.  Needs per_member_inputs = 1 (else FI_ESTATE); launches eagerly. */
fi_status fi_run_batches(fi_dag* dag, const void* const* d_inputs, const int32_t* batches, void* const* d_outputs,
                         void* hip_stream);

/* One lane of that pass, on the caller's stream: only the launches of the members of `lane`
 * (fi_member_info.lane; lanes are 0 .. fi_dag_info.n_lanes - 1) run, for batches[m] images of each of
 * them; the entries of members of other lanes are ignored.  Lanes share no tensor and the call touches
 * no state of the handle, so calls for DIFFERENT lanes may be in flight at the same time, on different
 * streams and from different threads (two calls for one lane may not).  Needs per_member_inputs = 1. */
fi_status fi_run_lane(fi_dag* dag, int32_t lane, const void* const* d_inputs, const int32_t* batches,
                      void* const* d_outputs, void* hip_stream);

/* Same pass with every launch issued on hip_stream (lanes serialised) and a HIP
 * event between launches; ms[i] (host, n_launches floats) receives launch i's
 * elapsed milliseconds: the kernel's own time with the chip to itself.
 * Synchronises the stream. */
fi_status fi_profile(fi_dag* dag, const void* d_input, int32_t batch, void* const* d_outputs, void* hip_stream,
                     float* ms, int32_t n_ms);

/* Same pass issued exactly as fi_run issues it (Section 3: independent members
 * run side by side, here as concurrent lanes), with a HIP event after every
 * launch on the stream it went to.  Launch i occupies [begin_ms[i], end_ms[i]]
 * (host arrays, n >= n_launches floats each), in milliseconds since the pass
 * began: from the end of the previous launch on the same stream to its own
 * end.  Intervals of different lanes overlap.  Synchronises the stream. */
fi_status fi_timeline(fi_dag* dag, const void* d_input, int32_t batch, void* const* d_outputs, void* hip_stream,
                      float* begin_ms, float* end_ms, int32_t n);

/* Section V, "individual model swaps in a DAG" (Table IV): replaces member `slot`
 * by `model` without recompiling or reloading the rest.  The sub-graph of the
 * outgoing member is dropped, the newcomer's is compiled into the schedule, and
 * in a LOADED handle only the newcomer's packed weights travel to the device
 * (one copy, asynchronous on hip_stream) into the lowest free range of the weight
 * arena that holds them; every other member's weights stay where they are, and
 * their outputs keep their bits.  The handle may be BUILT (host work only) or
 * LOADED; no fi_run may be in flight on another stream.  `model` follows the rules
 * of fi_build_dag (borrowed; same weight dtype and input shape as the other
 * members; device layout required in FI_LOAD_PER_MODEL).  Fails, leaving the DAG
 * exactly as it was, with FI_EBUDGET when the new plan does not fit the loaded
 * allocation (fi_build_opts.swap_headroom_bytes reserves room at load) or
 * max_device_bytes, and with the fi_build_dag errors for a bad model. */
fi_status fi_swap_model(fi_dag* dag, int32_t slot, const fi_model_spec* model, void* hip_stream);

/* ---- manager-side scheduling (Section IV, "Manager"; Section V, consecutive swaps) ----
 * A set of models that does not fit the device at once is cut into batches that
 * each fit; every batch is compiled into its own DAG; the scheduler runs a fixed
 * number of iterations per DAG, swaps it out and takes the next, round robin. */

/* Batches in the caller's order, first fit: model m joins the current batch while
 * the batch's exact device footprint (fi_footprint) stays within budget_bytes.
 * group_of: host, n entries out (batch index of every model, non-decreasing);
 * n_groups: out.  FI_EBUDGET when a single model exceeds the budget. */
fi_status fi_partition(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, uint64_t budget_bytes,
                       int32_t* group_of, int32_t* n_groups);

typedef struct {
  int32_t iterations;   /* fi_run passes per DAG before it is swapped out (>= 1) */
  int32_t rounds;       /* round-robin rounds over all batches (>= 1) */
  int32_t overlap_load; /* 1: the next batch is loaded on an internal copy stream while the current one
                           computes, so two batches are resident at a time; 0: unload, then load */
  int32_t reserved;
} fi_sched_opts;

typedef struct {
  double build_ms;            /* compiling every batch (host, once) */
  double total_ms;            /* all rounds: loads, runs, unloads */
  double run_ms;              /* time spent waiting for the runs of a batch (incl. a load still in flight) */
  double swap_ms;             /* time spent in unload (+ the next load when not overlapped) */
  uint64_t peak_device_bytes; /* largest resident footprint (two batches with overlap_load) */
  int32_t n_loads, n_runs, n_groups, reserved;
} fi_sched_stats;

/* Compiles one DAG per batch (group_of as produced by fi_partition; any grouping
 * with every batch non-empty is accepted), then for `rounds` rounds visits the
 * batches in order: load, `iterations` x fi_run on hip_stream with the shared
 * d_input (device, as for fi_run), unload.  d_outputs: HOST array of n DEVICE
 * pointers indexed like `models`; model m's buffer holds the output of its last
 * run on return.  A single batch stays resident for all rounds.  With
 * opts->max_device_bytes set, FI_EBUDGET if the resident peak would exceed it.
 * Synchronous: returns after the last unload.  stats may be NULL. */
fi_status fi_round_robin(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, const int32_t* group_of,
                         int32_t n_groups, const fi_sched_opts* sched, const void* d_input, int32_t batch,
                         void* const* d_outputs, void* hip_stream, fi_sched_stats* stats);

/* ---- request aggregation (Section IV, "Manager": requests that arrive while the device
 * is busy are gathered per model into the next batch) ----
 * A server sits in front of a LOADED DAG built with per_member_inputs = 1.  Callers submit
 * single images for single members; every lane of the DAG has a worker thread (with a stream
 * of its own) that repeatedly takes up to max_batch waiting requests of each of its members,
 * runs ONE fi_run_lane pass and hands every request its output row.  The busier the device,
 * the larger the batches; a short model never waits for a long one.  While a server runs,
 * nothing else may use the DAG. */
typedef struct fi_server fi_server; /* opaque, owned by the library */

typedef struct {
  int32_t max_wait_us; /* when a request finds the server idle, wait this long for companions before
                          the pass starts (0 = start at once) */
  int32_t reserved;
} fi_server_opts;

typedef struct {
  uint64_t requests, passes;    /* requests served; lane passes (fi_run_lane) issued */
  uint64_t max_images_per_pass; /* most requests one lane pass carried (all members of the lane together) */
  double mean_images_per_pass;
  double mean_latency_ms, max_latency_ms; /* submit to output written, host clock */
  double busy_ms;               /* time with a pass in flight, summed over the lanes */
} fi_server_stats;

/* Allocates, through the DAG's allocator callbacks, one batch buffer of max_batch images and one of
 * max_batch output rows per member, and starts the worker on the current device.  opts may be NULL.
 * FI_ESTATE unless the DAG is LOADED and was built with per_member_inputs = 1. */
fi_status fi_server_start(fi_dag* dag, const fi_server_opts* opts, fi_server** out);
/* Queues one image for member `member`.  d_image: device, [in_h, in_w, in_c] in the weight dtype,
 * complete in memory before the call and untouched until fi_server_wait returns; d_output: device,
 * receives the member's output row (fp32, classes_m values).  Requests of one member are served in
 * order.  Thread-safe.  ticket: out, never 0. */
fi_status fi_server_submit(fi_server* srv, int32_t member, const void* d_image, void* d_output, uint64_t* ticket);
/* Blocks until the request's output is in d_output (the copy has completed).  Thread-safe.  Reports
 * the worker's error, if it met one, on this and every later call. */
fi_status fi_server_wait(fi_server* srv, uint64_t ticket);
fi_status fi_server_query(fi_server* srv, fi_server_stats* stats);
/* Section V, individual model swaps, under load: replaces member `slot` of the served DAG (fi_swap_model).
 * The requests already queued for the slot are served by the outgoing model first; then every lane
 * finishes its pass in flight, the swap re-plans the DAG (its lanes included) and new workers start.
 * Requests for the slot submitted while the call is in progress are refused with FI_ESTATE; requests
 * for the other members are accepted throughout and served before or after the swap.  Blocks until
 * the newcomer's weights are on the device.
 * `model` is borrowed as by fi_swap_model (until fi_destroy of the DAG).  Errors of fi_swap_model are
 * returned and leave the server as it was. */
fi_status fi_server_swap(fi_server* srv, int32_t slot, const fi_model_spec* model);
/* Serves what is queued, joins the worker, releases the buffers and the handle; the DAG stays LOADED. */
fi_status fi_server_stop(fi_server* srv);

/* Sections I and III (problem statement: models are swapped in and out of device
 * memory many times a day; C3, low overhead): the swap-out half.  Synchronises the
 * device, returns the one allocation (through fi_build_opts.dev_free when given);
 * the handle goes back to BUILT with its plan and pinned image intact, so the same
 * DAG can be loaded again without recompiling.  FI_ESTATE unless LOADED. */
fi_status fi_unload(fi_dag* dag);
/* Same passages: the end of a DAG's life.  Unloads if needed, frees the pinned image
 * and the plan; the specs and host blobs the handle borrowed are the caller's again.
 * NULL is allowed. */
void fi_destroy(fi_dag* dag);

const char* fi_last_error(void); /* thread-local, valid until the next call on this thread */
const char* fi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FUSEDINF_H */
