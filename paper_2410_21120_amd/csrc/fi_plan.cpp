// Host-side analysis of one member model: validation, shape inference, the
// device (packed) weight layout, and the canonical -> packed conversion.
//
// Packed layout of a member (all offsets 256-byte aligned, node order):
//   conv       w [cout][kh][kw][Cp]  each row zero-padded to Kp elements, model dtype
//   depthwise  w [kh][kw][Cp]        (tap-major, channel innermost), model dtype
//   fc         w [cout][H][W][Cp]    i.e. the input tensor's NHWC storage order, row padded to Kp (fp32 weights);
//              bf16 weights: the same rows cut into the blocks the matrix cores consume, so that a wave's load is
//              one contiguous kilobyte: [cout/32][Kp/16][64][8] where entry (t, s, l) holds elements
//              s*16 + (l/32)*8 .. +8 of row t*32 + l%32 (rows past cout are zero)
//   bias       fp32 [Cop]
// Cp rounds channels up to 8 for bf16 weights (16-byte vectors along C) and to 1 for
// fp32.  Kp rounds the row up to 32 elements for bf16 so a reduction tile never straddles
// the end of a row; pad weights are zero, so whatever finite activation sits in a padded
// channel contributes nothing.
#include <cstdarg>
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <vector>

#include "fi_internal.h"

namespace fi {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
const char* last_error() { return g_err; }

static inline int32_t round_up(int32_t v, int32_t g) { return (v + g - 1) / g * g; }

fi_status analyze_model(const fi_model_spec& m, ModelPlan& out) {
  const char* nm = m.name ? m.name : "?";
  if (m.dtype != FI_F32 && m.dtype != FI_BF16) { set_error("model %s: bad dtype %d", nm, m.dtype); return FI_EINVAL; }
  if (m.act_dtype != FI_F32 && m.act_dtype != FI_BF16) { set_error("model %s: bad act_dtype %d", nm, m.act_dtype); return FI_EINVAL; }
  if (m.dtype == FI_F32 && m.act_dtype != FI_F32) { set_error("model %s: fp32 weights need fp32 activations", nm); return FI_EINVAL; }
  if (m.n_layers <= 0 || !m.layers) { set_error("model %s: no layers", nm); return FI_EINVAL; }
  if (m.in_c <= 0 || m.in_h <= 0 || m.in_w <= 0) { set_error("model %s: bad input shape", nm); return FI_EINVAL; }
  if (m.in_c > kMaxChannels || m.in_h > kMaxSide || m.in_w > kMaxSide || (int64_t)m.in_c * m.in_h * m.in_w > kMaxElems) {
    set_error("model %s: input larger than %d channels, %d x %d pixels or %d elements per image", nm, kMaxChannels, kMaxSide, kMaxSide, kMaxElems);
    return FI_EUNSUPPORTED; }
  if (m.output_node < 0 || m.output_node >= m.n_layers) { set_error("model %s: output_node out of range", nm); return FI_EINVAL; }
  const int32_t g = m.dtype == FI_BF16 ? 8 : 1;
  const int32_t kg = m.dtype == FI_BF16 ? 32 : 1;
  const uint64_t wsz = m.dtype == FI_BF16 ? 2 : 4;
  out.cgran = g;
  out.in_cp = round_up(m.in_c, g);
  if (m.dtype == FI_BF16 && m.in_c <= 4) {
    // An RGB-like input padded to 8 channels would make five eighths of the first convolution's
    // reduction zeros; when only convolutions read the input it is staged with 4 channels and the
    // kernels gather each 8-element vector from two neighbouring filter taps.
    bool only_convs = true;
    for (int32_t i = 0; i < m.n_layers; ++i)
      if (m.layers[i].input == FI_INPUT && m.layers[i].op != FI_CONV2D) only_convs = false;
    if (only_convs) out.in_cp = 4;
  }
  out.nodes.assign((size_t)m.n_layers, Node{});
  uint64_t off = 0;
  for (int32_t i = 0; i < m.n_layers; ++i) {
    const fi_layer_spec& L = m.layers[i];
    Node& n = out.nodes[(size_t)i];
    n.index = i; n.op = L.op; n.act = L.act; n.input = L.input; n.residual = L.residual;
    if (L.input != FI_INPUT && (L.input < 0 || L.input >= i)) {
      set_error("model %s node %d: input %d is not an earlier node (cycle or dangling edge)", nm, i, L.input);
      return FI_EINVAL;
    }
    if (L.residual != FI_NO_RESIDUAL && (L.residual < 0 || L.residual >= i)) {
      set_error("model %s node %d: residual %d is not an earlier node", nm, i, L.residual);
      return FI_EINVAL;
    }
    if (L.act < FI_ACT_NONE || L.act > FI_ACT_SIGMOID) { set_error("model %s node %d: bad activation", nm, i); return FI_EINVAL; }
    // Every size field is bounded before any arithmetic on it, so that nothing below can overflow.
    if (L.cin < 0 || L.cin > kMaxElems || L.cout < 0 || L.cout > kMaxChannels || L.kh < 0 || L.kh > kMaxWindow ||
        L.kw < 0 || L.kw > kMaxWindow || L.stride < 0 || L.stride > kMaxWindow || L.pad < 0 || L.pad > kMaxWindow ||
        L.groups < 0 || L.groups > kMaxChannels || L.c_first < 0 || L.c_first > kMaxChannels) {
      set_error("model %s node %d: a size field is negative or beyond the supported range", nm, i); return FI_EINVAL; }
    if (L.input == FI_INPUT) { n.C = m.in_c; n.H = m.in_h; n.W = m.in_w; n.Cp = out.in_cp; }
    else { const Node& s = out.nodes[(size_t)L.input]; n.C = s.Co; n.H = s.Ho; n.W = s.Wo; n.Cp = s.Cop; }
    n.k = 1; n.kw = 1; n.stride = 1; n.pad = 0; n.pad_w = 0;
    switch (L.op) {
      case FI_CONV2D:
      case FI_DWCONV2D:
        if (L.kh < 1 || L.kw < 1 || L.stride < 1 || L.pad < 0 || L.cout < 1 ||
            (L.kh != L.kw && (L.op != FI_CONV2D || L.groups > 1))) {   // rectangular kernels: dense conv2d only
          set_error("model %s node %d: unsupported kernel geometry", nm, i); return FI_EUNSUPPORTED; }
        if (L.cin != n.C) { set_error("model %s node %d: cin %d != producer channels %d", nm, i, L.cin, n.C); return FI_EINVAL; }
        if (L.kh > 15 || L.kw > 15) { set_error("model %s node %d: kernels larger than 15x15 are not supported", nm, i); return FI_EUNSUPPORTED; }
        if (L.op == FI_DWCONV2D && L.cout != L.cin) { set_error("model %s node %d: depthwise needs cin == cout", nm, i); return FI_EINVAL; }
        if (L.groups > 1 && (L.op != FI_CONV2D || L.cin % L.groups || L.cout % L.groups)) {
          set_error("model %s node %d: %d groups do not divide cin %d and cout %d of a conv2d", nm, i, L.groups, L.cin, L.cout); return FI_EINVAL; }
        if (L.groups < 0) { set_error("model %s node %d: negative groups", nm, i); return FI_EINVAL; }
        n.k = L.kh; n.kw = L.kw; n.stride = L.stride; n.pad = L.pad; n.pad_w = L.pad; n.Co = L.cout;
        if (L.kh != L.kw) {   // a rectangular kernel is padded only along the dimensions it extends over
          n.pad = L.kh > 1 ? L.pad : 0;
          n.pad_w = L.kw > 1 ? L.pad : 0;
        }
        n.Ho = (n.H + 2 * n.pad - L.kh) / L.stride + 1;
        n.Wo = (n.W + 2 * n.pad_w - L.kw) / L.stride + 1;
        if (n.Ho < 1 || n.Wo < 1 || n.H + 2 * n.pad < L.kh || n.W + 2 * n.pad_w < L.kw) { set_error("model %s node %d: empty output", nm, i); return FI_EINVAL; }
        n.macs = (uint64_t)n.Ho * n.Wo * n.Co * (uint64_t)(L.op == FI_CONV2D ? n.C / (L.groups > 1 ? L.groups : 1) : 1) * L.kh * L.kw;
        n.groups = (L.op == FI_CONV2D && L.groups > 1) ? L.groups : 1;
        break;
      case FI_MAXPOOL2D:
      case FI_AVGPOOL2D:
        if (L.op == FI_AVGPOOL2D && L.ceil_mode) { set_error("model %s node %d: average pooling takes the floor output size only", nm, i); return FI_EUNSUPPORTED; }
        if (L.kh != L.kw || L.kh < 1 || L.stride < 1 || L.pad < 0 || 2 * L.pad > L.kh) {
          set_error("model %s node %d: unsupported pooling geometry", nm, i); return FI_EUNSUPPORTED; }
        n.k = L.kh; n.stride = L.stride; n.pad = L.pad; n.Co = n.C;
        n.Ho = (n.H + 2 * L.pad - L.kh) / L.stride + 1;
        n.Wo = (n.W + 2 * L.pad - L.kh) / L.stride + 1;
        if (n.Ho < 1 || n.Wo < 1 || n.H + 2 * L.pad < L.kh) { set_error("model %s node %d: empty output", nm, i); return FI_EINVAL; }
        if (L.ceil_mode) {  // round up, but the last window must start inside the input or its leading padding
          n.Ho = (n.H + 2 * L.pad - L.kh + L.stride - 1) / L.stride + 1;
          n.Wo = (n.W + 2 * L.pad - L.kh + L.stride - 1) / L.stride + 1;
          if ((n.Ho - 1) * L.stride >= n.H + L.pad) --n.Ho;
          if ((n.Wo - 1) * L.stride >= n.W + L.pad) --n.Wo;
        }
        if (L.act != FI_ACT_NONE || L.residual != FI_NO_RESIDUAL) { set_error("model %s node %d: pooling takes no activation/residual", nm, i); return FI_EUNSUPPORTED; }
        break;
      case FI_SLICE:
        if (L.input == FI_INPUT) { set_error("model %s node %d: slicing the model input is not supported", nm, i); return FI_EUNSUPPORTED; }
        if (L.c_first < 0 || L.cout < 1 || L.c_first + L.cout > n.C) { set_error("model %s node %d: slice [%d, %d) outside %d channels", nm, i, L.c_first, L.c_first + L.cout, n.C); return FI_EINVAL; }
        if (L.act != FI_ACT_NONE || L.residual != FI_NO_RESIDUAL) { set_error("model %s node %d: slice takes no activation/residual", nm, i); return FI_EUNSUPPORTED; }
        n.Co = L.cout; n.Ho = n.H; n.Wo = n.W;
        n.pad = L.c_first;   // first channel, carried in the pad field of the descriptor
        break;
      case FI_SHUFFLE:
        if (L.input == FI_INPUT) { set_error("model %s node %d: shuffling the model input is not supported", nm, i); return FI_EUNSUPPORTED; }
        if (L.groups < 1 || n.C % L.groups) { set_error("model %s node %d: %d groups do not divide %d channels", nm, i, L.groups, n.C); return FI_EINVAL; }
        if (L.act != FI_ACT_NONE || L.residual != FI_NO_RESIDUAL) { set_error("model %s node %d: shuffle takes no activation/residual", nm, i); return FI_EUNSUPPORTED; }
        n.Co = n.C; n.Ho = n.H; n.Wo = n.W;
        n.k = L.groups;      // groups, carried in the k field of the descriptor
        break;
      case FI_MUL: {
        if (L.residual == FI_NO_RESIDUAL || L.input == FI_INPUT) { set_error("model %s node %d: channel scaling needs a tensor and a gate node", nm, i); return FI_EINVAL; }
        const Node& gt = out.nodes[(size_t)L.residual];
        if (gt.Co != n.C || gt.Ho != 1 || gt.Wo != 1) { set_error("model %s node %d: the gate must be a 1x1 tensor with the input's %d channels", nm, i, n.C); return FI_EINVAL; }
        if (L.act != FI_ACT_NONE) { set_error("model %s node %d: channel scaling takes no activation", nm, i); return FI_EUNSUPPORTED; }
        n.Co = n.C; n.Ho = n.H; n.Wo = n.W;
        break;
      }
      case FI_CONCAT: {
        if (L.residual == FI_NO_RESIDUAL) { set_error("model %s node %d: concat needs a second source", nm, i); return FI_EINVAL; }
        const Node& b = out.nodes[(size_t)L.residual];
        if (L.input == FI_INPUT) { set_error("model %s node %d: concat of the model input is not supported", nm, i); return FI_EUNSUPPORTED; }
        if (b.Ho != n.H || b.Wo != n.W) { set_error("model %s node %d: concat sources differ in height or width", nm, i); return FI_EINVAL; }
        if (L.act != FI_ACT_NONE) { set_error("model %s node %d: concat takes no activation", nm, i); return FI_EUNSUPPORTED; }
        n.Co = n.C + b.Co; n.Ho = n.H; n.Wo = n.W;
        if (L.cout != n.Co) { set_error("model %s node %d: concat cout %d != %d + %d", nm, i, L.cout, n.C, b.Co); return FI_EINVAL; }
        break;
      }
      case FI_GLOBAL_AVGPOOL:
        n.Co = n.C; n.Ho = 1; n.Wo = 1;
        if (L.act != FI_ACT_NONE || L.residual != FI_NO_RESIDUAL) { set_error("model %s node %d: pooling takes no activation/residual", nm, i); return FI_EUNSUPPORTED; }
        break;
      case FI_FC:
        if (L.cout < 1) { set_error("model %s node %d: bad cout", nm, i); return FI_EINVAL; }
        if ((int64_t)L.cin != (int64_t)n.C * n.H * n.W) { set_error("model %s node %d: fc cin %d != %d*%d*%d", nm, i, L.cin, n.C, n.H, n.W); return FI_EINVAL; }
        n.Co = L.cout; n.Ho = 1; n.Wo = 1;
        n.macs = (uint64_t)L.cout * L.cin;
        break;
      case FI_SOFTMAX:
        if (n.H != 1 || n.W != 1) { set_error("model %s node %d: softmax needs a 1x1 input", nm, i); return FI_EUNSUPPORTED; }
        if (L.act != FI_ACT_NONE || L.residual != FI_NO_RESIDUAL) { set_error("model %s node %d: softmax takes no activation/residual", nm, i); return FI_EUNSUPPORTED; }
        n.Co = n.C; n.Ho = 1; n.Wo = 1;
        break;
      default:
        set_error("model %s node %d: unknown op %d", nm, i, L.op);
        return FI_EUNSUPPORTED;
    }
    if (n.Co > kMaxChannels || (int64_t)round_up(n.Co, g) * n.Ho * n.Wo > kMaxElems) {
      set_error("model %s node %d: output larger than %d channels or %d elements per image", nm, i, kMaxChannels, kMaxElems);
      return FI_EUNSUPPORTED; }
    n.Cop = round_up(n.Co, g);
    if (L.residual != FI_NO_RESIDUAL && L.op != FI_CONCAT && L.op != FI_MUL) {
      const Node& r = out.nodes[(size_t)L.residual];
      if (r.Co != n.Co || r.Ho != n.Ho || r.Wo != n.Wo) {
        set_error("model %s node %d: residual shape mismatch", nm, i); return FI_EINVAL; }
    }
    // packed weight placement
    n.w_rel = n.b_rel = kNone;
    uint64_t wbytes = 0;
    if (L.op == FI_CONV2D) { n.Kp = round_up(n.k * n.kw * n.Cp, kg); wbytes = (uint64_t)n.Co * n.Kp * wsz; }
    else if (L.op == FI_FC) { n.Kp = round_up(n.H * n.W * n.Cp, kg); wbytes = (uint64_t)(m.dtype == FI_BF16 ? round_up(n.Co, 32) : n.Co) * n.Kp * wsz; }
    else if (L.op == FI_DWCONV2D) { n.Kp = n.k * n.k; wbytes = (uint64_t)n.k * n.k * n.Cp * wsz; }
    if (wbytes) {
      n.w_rel = off; off = align_up(off + wbytes);
      n.b_rel = off; off = align_up(off + (uint64_t)n.Cop * 4);
      // canonical blob bounds
      const uint64_t cw = (L.op == FI_CONV2D ? (uint64_t)n.Co * (n.C / (L.groups > 1 ? L.groups : 1)) * n.k * n.kw
                           : L.op == FI_FC  ? (uint64_t)n.Co * L.cin : (uint64_t)n.Co * n.k * n.k) * wsz;
      if (!m.weights_packed && m.weights &&
          (L.w_off > m.weight_bytes || cw > m.weight_bytes - L.w_off ||
           L.b_off > m.weight_bytes || (uint64_t)n.Co * 4 > m.weight_bytes - L.b_off)) {
        set_error("model %s node %d: weight/bias offsets run past the blob", nm, i); return FI_EINVAL; }
    }
  }
  // stored dtype of every node: fp32 for the output node, softmax nodes and an fc that
  // feeds only softmax nodes; the member's act_dtype otherwise
  for (int32_t i = 0; i < m.n_layers; ++i) {
    Node& n = out.nodes[(size_t)i];
    n.out_dtype = m.act_dtype;
    n.is_output = (i == m.output_node);
    if (n.is_output || n.op == FI_SOFTMAX) n.out_dtype = FI_F32;
    if (n.op == FI_FC) {
      bool any = false, all_sm = true;
      for (int32_t j = i + 1; j < m.n_layers; ++j)
        if (m.layers[j].input == i || m.layers[j].residual == i) { any = true; if (m.layers[j].op != FI_SOFTMAX) all_sm = false; }
      if (any && all_sm) n.out_dtype = FI_F32;
    }
    if (n.op == FI_SOFTMAX && out.nodes[(size_t)n.input].out_dtype != FI_F32) {
      set_error("model %s node %d: softmax input must be an fc that feeds only softmax", nm, i); return FI_EUNSUPPORTED; }
    if (n.out_dtype == FI_F32 && m.act_dtype != FI_F32 && !n.is_output && n.op != FI_SOFTMAX && n.op != FI_FC) {
      set_error("model %s node %d: internal error (dtype rule)", nm, i); return FI_EINVAL; }
  }
  // an fp32-stored fc/softmax value consumed by anything but softmax/nothing is not supported
  for (int32_t j = 0; j < m.n_layers; ++j) {
    const fi_layer_spec& L = m.layers[j];
    for (int32_t src : {L.input, L.residual}) {
      if (src < 0) continue;
      const Node& s = out.nodes[(size_t)src];
      if (s.out_dtype == FI_F32 && m.act_dtype != FI_F32 && L.op != FI_SOFTMAX) {
        set_error("model %s node %d: consumes the fp32 output node %d", nm, j, src); return FI_EUNSUPPORTED; }
    }
  }
  out.packed_bytes = align_up(off ? off : kAlign);
  return FI_OK;
}

// Canonical (OIHW, model dtype) -> packed.  Pure data movement: elements are copied, never
// converted, and padding is zero-filled.
template <typename T>
static void pack_typed(const fi_model_spec& m, const ModelPlan& p, uint8_t* dst8) {
  const uint8_t* src = static_cast<const uint8_t*>(m.weights);
  std::memset(dst8, 0, (size_t)p.packed_bytes);
  for (int32_t i = 0; i < m.n_layers; ++i) {
    const Node& n = p.nodes[(size_t)i];
    if (n.w_rel == kNone) continue;
    const fi_layer_spec& L = m.layers[i];
    const T* w = reinterpret_cast<const T*>(src + L.w_off);
    T* d = reinterpret_cast<T*>(dst8 + n.w_rel);
    const int32_t kk = n.op == FI_CONV2D ? n.k * n.kw : n.k * n.k;
    if (n.op == FI_CONV2D) {
      // A grouped convolution becomes a dense one whose weight rows are zero outside the row's own
      // group of input channels (block-diagonal): the kernels need no notion of groups.
      const int32_t G = L.groups > 1 ? L.groups : 1;
      const int32_t cg = n.C / G, og = n.Co / G;
      for (int32_t o = 0; o < n.Co; ++o) {
        const T* wo = w + (size_t)o * cg * kk;
        T* dorow = d + (size_t)o * n.Kp;
        const int32_t c0 = (o / og) * cg;   // first input channel of this row's group
        if (kk == 1) { std::memcpy(dorow + c0, wo, (size_t)cg * sizeof(T)); continue; }
        for (int32_t t = 0; t < kk; ++t) {
          T* dt = dorow + (size_t)t * n.Cp + c0;
          for (int32_t c = 0; c < cg; ++c) dt[c] = wo[(size_t)c * kk + t];
        }
      }
    } else if (n.op == FI_FC) {
      // canonical column index runs over (c, h, w); packed over (h, w, c) with stride Cp
      const int32_t HW = n.H * n.W;
      std::vector<T> row((size_t)n.Kp);
      for (int32_t o = 0; o < n.Co; ++o) {
        const T* wr = w + (size_t)o * n.C * HW;
        T* dr = sizeof(T) == 2 ? row.data() : d + (size_t)o * n.Kp;
        if (sizeof(T) == 2) std::fill(row.begin(), row.end(), T(0));
        if (HW == 1) std::memcpy(dr, wr, (size_t)n.C * sizeof(T));
        else
          for (int32_t q = 0; q < HW; ++q) {
            T* dq = dr + (size_t)q * n.Cp;
            for (int32_t c = 0; c < n.C; ++c) dq[c] = wr[(size_t)c * HW + q];
          }
        if (sizeof(T) == 2) {   // bf16: scatter the row into its 32-row tile, 8 elements (16 bytes) per (step, lane)
          const size_t steps = (size_t)n.Kp / 16;
          T* tile = d + (size_t)(o / 32) * steps * 64 * 8;
          for (size_t k8 = 0; k8 < (size_t)n.Kp / 8; ++k8)
            std::memcpy(tile + ((k8 / 2) * 64 + (k8 % 2) * 32 + (size_t)(o % 32)) * 8, dr + k8 * 8, 8 * sizeof(T));
        }
      }
    } else {  // depthwise: [c][0][r][s] -> [r][s][c]
      for (int32_t t = 0; t < kk; ++t)
        for (int32_t c = 0; c < n.C; ++c) d[(size_t)t * n.Cp + c] = w[(size_t)c * kk + t];
    }
    std::memcpy(dst8 + n.b_rel, src + L.b_off, (size_t)n.Co * 4);
  }
}

void pack_model(const fi_model_spec& m, const ModelPlan& p, uint8_t* dst) {
  if (m.dtype == FI_BF16) pack_typed<uint16_t>(m, p, dst);
  else pack_typed<uint32_t>(m, p, dst);
}

}  // namespace fi
