// CPU oracle for the fused multi-model CNN forward pass.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, single-threaded, obviously-correct definition that the
// GPU library is checked against.  Only tests, the smoke check and the benchmark's
// cpu_baseline leg may call it; the product path never does, and this file shares
// no code, header, table or helper with the GPU library.
//
// What it computes.  The paper (FusedInf, Section IV "System Design", Algorithm 1
// and the correctness / privacy properties C1 and C4 of Section III) states that a
// fused DAG is the disjoint union of the member models' graphs and that every
// member's output is exactly what the member produces alone: fusion changes how
// models are loaded and launched, never what a node computes.  Each node evaluates
// phi(sum_j u_j * x_j) (Algorithm 1, inference loop): a weighted sum followed by
// the node's activation.  The oracle therefore is the plain definition: each
// member model's own forward pass, alone, node by node in topological order.  It
// never builds a DAG, never sees levels, arenas, groups or NHWC.
//
// The paper delegates the layer arithmetic to a vendor library, so the layer
// definitions are the textbook ones:
//   conv2d      cross-correlation, zero padding, square kernel k, stride s, pad p,
//               Ho = floor((H + 2p - k) / s) + 1,
//               y[n,o,i,j] = b[o] + sum_c sum_r sum_t x[n,c,i*s-p+r,j*s-p+t] * w[o,c,r,t]
//   depthwise   same with one input channel per output channel
//   residual    z = act(conv(x) + b + skip): the skip is added before the activation
//   ReLU max(0,x); ReLU6 min(max(0,x),6)
//   maxpool     max over the in-range taps only (padding behaves as -inf), floor size
//   global avg  (sum_{h,w} x) / (H*W)
//   FC          y[n,o] = b[o] + sum_i x[n,i] * W[o,i], i running over (c,h,w)
//   softmax     p_k = exp(z_k - max z) / sum_j exp(z_j - max z)
// Tensors are logical NCHW, weights OIHW.  Every sum is accumulated in `acc_t`
// (float by default; build with -DORC_ACC=double for the cross-check build) in
// the fixed order c -> r -> t starting from the bias, with no FMA contraction.
//
// Storage-rounding mode ("mode S").  With round_storage != 0 the value a node
// hands to its consumers is rounded to bf16 (round-to-nearest-even) exactly where
// a bf16 executor stores bf16: after conv / depthwise (after bias, residual and
// activation), after global-average pooling, and after an FC whose value is
// consumed by another FC.  The model's output node, softmax nodes and an FC that
// feeds only a softmax keep fp32.  With round_storage == 0 ("mode F") activations
// stay fp32 throughout.
//
// Pins (tests, not marked gpu): brute-force scatter-form and im2col x matmul
// convolutions, a library convolution in fp64, delta/identity kernels, closed
// forms for all-ones convolution, ramp pooling, softmax; linearity; BN-fold
// identity; FC == 1x1 conv == 7x7 valid conv; the double-accumulation build.
// Real-accuracy numbers (ImageNet top-1/top-5 of trained models): parity unpinned
// and out of scope: neither the dataset nor trained weights are available.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

#ifndef ORC_ACC
#define ORC_ACC float
#endif
typedef ORC_ACC acc_t;

extern "C" {

enum { ORC_CONV = 0, ORC_DWCONV = 1, ORC_MAXPOOL = 2, ORC_GAP = 3, ORC_FC = 4, ORC_SOFTMAX = 5, ORC_CONCAT = 6, ORC_AVGPOOL = 7, ORC_MUL = 8, ORC_SLICE = 9, ORC_SHUFFLE = 10 };
enum { ORC_NONE = 0, ORC_RELU = 1, ORC_RELU6 = 2, ORC_HARDSWISH = 3, ORC_HARDSIGMOID = 4, ORC_SILU = 5, ORC_SIGMOID = 6 };
enum { ORC_F32 = 0, ORC_BF16 = 1 };

// One node of a model's layer graph (the oracle's own description format).
struct orc_layer {
  int32_t op;
  int32_t act;
  int32_t input;     // node index, -1 = model input
  int32_t residual;  // node index added before the activation, < 0 = none; concat: the second source
  int32_t cin, cout, k, stride, pad;
  int32_t ceil_mode; // pooling: output size rounds up
  int64_t w_off, b_off;  // byte offsets into the canonical weight blob
  int32_t groups;        // conv: number of channel groups (0 or 1 = dense); shuffle: number of groups
  int32_t c_first;       // slice: first channel taken
  int32_t kw;            // conv: kernel width when it differs from the height k (0 = square); the padding
                         // then applies only along a dimension the kernel extends over (size > 1)
  int32_t reserved;
};

// ---- scalar helpers -------------------------------------------------------

// fp32 -> nearest bf16 (ties to even), returned as fp32.
float orc_bf16_round(float v) {
  uint32_t u;
  std::memcpy(&u, &v, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return v;  // inf / nan unchanged
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  float r;
  std::memcpy(&r, &u, 4);
  return r;
}

static inline float bf16_bits_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float r;
  std::memcpy(&r, &u, 4);
  return r;
}

void orc_round_bf16(float* y, int64_t n) {
  for (int64_t i = 0; i < n; ++i) y[i] = orc_bf16_round(y[i]);
}

void orc_activate(float* y, int64_t n, int act) {
  if (act == ORC_RELU) {
    for (int64_t i = 0; i < n; ++i) y[i] = y[i] > 0.0f ? y[i] : 0.0f;
  } else if (act == ORC_RELU6) {
    for (int64_t i = 0; i < n; ++i) {
      float v = y[i] > 0.0f ? y[i] : 0.0f;
      y[i] = v < 6.0f ? v : 6.0f;
    }
  } else if (act == ORC_HARDSWISH || act == ORC_HARDSIGMOID) {
    // hard sigmoid h(v) = min(max(v + 3, 0), 6) / 6; hard swish = v * h(v)
    for (int64_t i = 0; i < n; ++i) {
      float t = y[i] + 3.0f;
      t = t > 0.0f ? t : 0.0f;
      t = t < 6.0f ? t : 6.0f;
      y[i] = act == ORC_HARDSWISH ? y[i] * t / 6.0f : t / 6.0f;
    }
  } else if (act == ORC_SILU || act == ORC_SIGMOID) {
    // logistic sigmoid s(v) = 1 / (1 + exp(-v)); SiLU = v * s(v)
    for (int64_t i = 0; i < n; ++i) {
      const float sg = 1.0f / (1.0f + std::exp(-y[i]));
      y[i] = act == ORC_SILU ? y[i] * sg : sg;
    }
  }
}

// Per-(image, channel) gate: y[n,c,h,w] = x[n,c,h,w] * g[n,c]  (squeeze-and-excitation's rescaling).
void orc_channel_scale(const float* x, const float* g, int N, int C, int H, int W, float* y) {
  const int64_t hw = (int64_t)H * W;
  for (int64_t nc = 0; nc < (int64_t)N * C; ++nc)
    for (int64_t i = 0; i < hw; ++i) y[nc * hw + i] = x[nc * hw + i] * g[nc];
}

void orc_add(float* y, const float* skip, int64_t n) {
  for (int64_t i = 0; i < n; ++i) y[i] = y[i] + skip[i];
}

static inline int out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }
// Output size that rounds up: windows may hang over the far edge, but the last one must still
// start inside the input or its leading padding.
static inline int out_size_ceil(int in, int k, int s, int p) {
  int out = (in + 2 * p - k + s - 1) / s + 1;
  if ((out - 1) * s >= in + p) --out;
  return out;
}

// ---- layers ---------------------------------------------------------------

// Accumulate one filter tap into an output plane: for every output pixel whose
// tap (r,t) lands inside the image, plane += wv * x.  Every output element sees
// its taps in the order the caller iterates (c, r, t).
static void tap_accumulate(acc_t* plane, const float* xc, float wv, int H, int W, int Ho, int Wo,
                           int s, int p, int r, int t) {
  for (int i = 0; i < Ho; ++i) {
    const int ih = i * s - p + r;
    if (ih < 0 || ih >= H) continue;
    const float* xrow = xc + (int64_t)ih * W;
    acc_t* prow = plane + (int64_t)i * Wo;
    // columns j with 0 <= j*s - p + t < W
    const int jlo = (p - t > 0) ? (p - t + s - 1) / s : 0;
    int jhi = (W - 1 + p - t >= 0) ? (W - 1 + p - t) / s : -1;
    if (jhi > Wo - 1) jhi = Wo - 1;
    const float* xs = xrow - p + t;
    for (int j = jlo; j <= jhi; ++j) prow[j] = prow[j] + (acc_t)wv * (acc_t)xs[j * s];
  }
}

// y[n,o,i,j] = b[o] + sum_c sum_r sum_t x[n,c,i*s-p+r,j*s-p+t] * w[o,c,r,t]
void orc_conv2d(const float* x, int N, int C, int H, int W, const float* w, const float* b, int O,
                int k, int s, int p, float* y) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
  std::vector<acc_t> plane((size_t)Ho * Wo);
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < O; ++o) {
      for (size_t q = 0; q < plane.size(); ++q) plane[q] = (acc_t)(b ? b[o] : 0.0f);
      for (int c = 0; c < C; ++c)
        for (int r = 0; r < k; ++r)
          for (int t = 0; t < k; ++t)
            tap_accumulate(plane.data(), x + ((int64_t)n * C + c) * H * W,
                           w[(((int64_t)o * C + c) * k + r) * k + t], H, W, Ho, Wo, s, p, r, t);
      float* yo = y + ((int64_t)n * O + o) * Ho * Wo;
      for (size_t q = 0; q < plane.size(); ++q) yo[q] = (float)plane[q];
    }
}

// Rectangular kernel, separate paddings: the definition written out per output element,
// y[n,o,i,j] = b[o] + sum_c sum_r sum_t x[n,c,i*s-ph+r,j*s-pw+t] * w[o,c,r,t], out-of-range x = 0.
void orc_conv2d_rect(const float* x, int N, int C, int H, int W, const float* w, const float* b, int O,
                     int kh, int kw, int s, int ph, int pw, float* y) {
  const int Ho = out_size(H, kh, s, ph), Wo = out_size(W, kw, s, pw);
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < O; ++o)
      for (int i = 0; i < Ho; ++i)
        for (int j = 0; j < Wo; ++j) {
          acc_t sum = (acc_t)(b ? b[o] : 0.0f);
          for (int c = 0; c < C; ++c)
            for (int r = 0; r < kh; ++r)
              for (int t = 0; t < kw; ++t) {
                const int ih = i * s - ph + r, iw = j * s - pw + t;
                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                sum = sum + (acc_t)w[(((int64_t)o * C + c) * kh + r) * kw + t] * (acc_t)x[(((int64_t)n * C + c) * H + ih) * W + iw];
              }
          y[(((int64_t)n * O + o) * Ho + i) * Wo + j] = (float)sum;
        }
}

// Grouped convolution: output channel o belongs to group g = o / (O/G) and sees only the input channels
// [g*C/G, (g+1)*C/G); w is [O][C/G][k][k].  G == 1 is orc_conv2d, G == C == O is the depthwise case.
void orc_conv2d_grouped(const float* x, int N, int C, int H, int W, const float* w, const float* b, int O,
                        int k, int s, int p, int G, float* y) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
  const int cg = C / G, og = O / G;
  std::vector<acc_t> plane((size_t)Ho * Wo);
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < O; ++o) {
      const int g = o / og;
      for (size_t q = 0; q < plane.size(); ++q) plane[q] = (acc_t)(b ? b[o] : 0.0f);
      for (int c = 0; c < cg; ++c)
        for (int r = 0; r < k; ++r)
          for (int t = 0; t < k; ++t)
            tap_accumulate(plane.data(), x + ((int64_t)n * C + g * cg + c) * H * W,
                           w[(((int64_t)o * cg + c) * k + r) * k + t], H, W, Ho, Wo, s, p, r, t);
      float* yo = y + ((int64_t)n * O + o) * Ho * Wo;
      for (size_t q = 0; q < plane.size(); ++q) yo[q] = (float)plane[q];
    }
}

// depthwise: y[n,c,i,j] = b[c] + sum_r sum_t x[n,c,i*s-p+r,j*s-p+t] * w[c,0,r,t]
void orc_dwconv2d(const float* x, int N, int C, int H, int W, const float* w, const float* b,
                  int k, int s, int p, float* y) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
  std::vector<acc_t> plane((size_t)Ho * Wo);
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      for (size_t q = 0; q < plane.size(); ++q) plane[q] = (acc_t)(b ? b[c] : 0.0f);
      for (int r = 0; r < k; ++r)
        for (int t = 0; t < k; ++t)
          tap_accumulate(plane.data(), x + ((int64_t)n * C + c) * H * W,
                         w[((int64_t)c * k + r) * k + t], H, W, Ho, Wo, s, p, r, t);
      float* yo = y + ((int64_t)n * C + c) * Ho * Wo;
      for (size_t q = 0; q < plane.size(); ++q) yo[q] = (float)plane[q];
    }
}

void orc_maxpool2d_ex(const float* x, int N, int C, int H, int W, int k, int s, int p, int ceil_mode, float* y);
void orc_maxpool2d(const float* x, int N, int C, int H, int W, int k, int s, int p, float* y) {
  orc_maxpool2d_ex(x, N, C, H, W, k, s, p, 0, y);
}

// Max over the taps that fall inside the image (padding and overhang are never candidates).
void orc_maxpool2d_ex(const float* x, int N, int C, int H, int W, int k, int s, int p, int ceil_mode, float* y) {
  const int Ho = ceil_mode ? out_size_ceil(H, k, s, p) : out_size(H, k, s, p);
  const int Wo = ceil_mode ? out_size_ceil(W, k, s, p) : out_size(W, k, s, p);
  for (int64_t nc = 0; nc < (int64_t)N * C; ++nc) {
    const float* xc = x + nc * H * W;
    float* yc = y + nc * Ho * Wo;
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        float m = -std::numeric_limits<float>::infinity();
        for (int r = 0; r < k; ++r)
          for (int t = 0; t < k; ++t) {
            const int ih = i * s - p + r, iw = j * s - p + t;
            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
            const float v = xc[(int64_t)ih * W + iw];
            if (v > m) m = v;
          }
        yc[(int64_t)i * Wo + j] = m;
      }
  }
}

// Average pooling, floor output size: the in-range taps of the window summed, divided by the full
// window area k*k (zero padding counts as zeros).
void orc_avgpool2d(const float* x, int N, int C, int H, int W, int k, int s, int p, float* y) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
  for (int64_t nc = 0; nc < (int64_t)N * C; ++nc) {
    const float* xc = x + nc * H * W;
    float* yc = y + nc * Ho * Wo;
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        acc_t sum = 0;
        for (int r = 0; r < k; ++r)
          for (int t = 0; t < k; ++t) {
            const int ih = i * s - p + r, iw = j * s - p + t;
            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
            sum += (acc_t)xc[(int64_t)ih * W + iw];
          }
        yc[(int64_t)i * Wo + j] = (float)(sum / (acc_t)(k * k));
      }
  }
}

// Channel slice: planes [first, first + count) of every image.
void orc_slice(const float* x, int N, int C, int H, int W, int first, int count, float* y) {
  const int64_t hw = (int64_t)H * W;
  for (int n = 0; n < N; ++n)
    for (int64_t i = 0; i < count * hw; ++i) y[(int64_t)n * count * hw + i] = x[((int64_t)n * C + first) * hw + i];
}

// Channel shuffle with G groups: the channels seen as a G x (C/G) matrix are transposed, i.e.
// output channel i*G + g is input channel g*(C/G) + i.
void orc_channel_shuffle(const float* x, int N, int C, int H, int W, int G, float* y) {
  const int64_t hw = (int64_t)H * W;
  const int per = C / G;
  for (int n = 0; n < N; ++n)
    for (int g = 0; g < G; ++g)
      for (int i = 0; i < per; ++i) {
        const float* src = x + ((int64_t)n * C + g * per + i) * hw;
        float* dst = y + ((int64_t)n * C + i * G + g) * hw;
        for (int64_t q = 0; q < hw; ++q) dst[q] = src[q];
      }
}

// Channel concatenation (NCHW): image n of y holds a's Ca planes, then b's Cb planes.
void orc_concat(const float* a, int Ca, const float* b, int Cb, int N, int H, int W, float* y) {
  const int64_t hw = (int64_t)H * W;
  for (int n = 0; n < N; ++n) {
    float* yn = y + (int64_t)n * (Ca + Cb) * hw;
    for (int64_t i = 0; i < Ca * hw; ++i) yn[i] = a[(int64_t)n * Ca * hw + i];
    for (int64_t i = 0; i < Cb * hw; ++i) yn[Ca * hw + i] = b[(int64_t)n * Cb * hw + i];
  }
}

void orc_global_avgpool(const float* x, int N, int C, int H, int W, float* y) {
  for (int64_t nc = 0; nc < (int64_t)N * C; ++nc) {
    acc_t sum = 0;
    for (int q = 0; q < H * W; ++q) sum = sum + (acc_t)x[nc * H * W + q];
    y[nc] = (float)(sum / (acc_t)(H * W));
  }
}

void orc_fc(const float* x, int N, int I, const float* w, const float* b, int O, float* y) {
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < O; ++o) {
      acc_t sum = (acc_t)(b ? b[o] : 0.0f);
      for (int i = 0; i < I; ++i) sum = sum + (acc_t)w[(int64_t)o * I + i] * (acc_t)x[(int64_t)n * I + i];
      y[(int64_t)n * O + o] = (float)sum;
    }
}

void orc_softmax(const float* z, int N, int K, float* p) {
  for (int n = 0; n < N; ++n) {
    const float* zr = z + (int64_t)n * K;
    float* pr = p + (int64_t)n * K;
    float m = zr[0];
    for (int q = 1; q < K; ++q)
      if (zr[q] > m) m = zr[q];
    acc_t sum = 0;
    for (int q = 0; q < K; ++q) {
      pr[q] = std::exp(zr[q] - m);
      sum = sum + (acc_t)pr[q];
    }
    for (int q = 0; q < K; ++q) pr[q] = (float)((acc_t)pr[q] / sum);
  }
}

// lowest index attaining the row maximum
void orc_top1(const float* z, int N, int K, int32_t* idx) {
  for (int n = 0; n < N; ++n) {
    int best = 0;
    for (int q = 1; q < K; ++q)
      if (z[(int64_t)n * K + q] > z[(int64_t)n * K + best]) best = q;
    idx[n] = best;
  }
}

// ---- whole model ----------------------------------------------------------

static std::vector<float> read_tensor(const uint8_t* blob, int64_t off, int64_t n, int dtype) {
  std::vector<float> v((size_t)n);
  if (dtype == ORC_F32) {
    std::memcpy(v.data(), blob + off, (size_t)n * 4);
  } else {
    const uint16_t* b = reinterpret_cast<const uint16_t*>(blob + off);
    for (int64_t i = 0; i < n; ++i) v[(size_t)i] = bf16_bits_to_f32(b[i]);
  }
  return v;
}

// Forward pass of ONE model, alone.  x: logical [N,C,H,W] fp32.  `output_node` is
// the model's output (it keeps fp32 in storage-rounding mode); out receives the
// value of node `return_node` as handed to its consumers ([N, cout] for
// FC/softmax/GAP, NCHW otherwise); out_cap is its capacity in floats.  Returns the number of floats
// written, or a negative code: -1 bad graph, -2 shape mismatch, -3 out too small.
int64_t orc_run_model(const orc_layer* layers, int n_layers, int output_node, const void* blob_v,
                      int dtype, const float* x, int N, int C, int H, int W, int round_storage,
                      int return_node, float* out, int64_t out_cap) {
  const uint8_t* blob = static_cast<const uint8_t*>(blob_v);
  if (n_layers <= 0 || output_node < 0 || output_node >= n_layers) return -1;
  if (return_node < 0 || return_node >= n_layers) return -1;
  struct T { std::vector<float> v; int c, h, w; };
  std::vector<T> val((size_t)n_layers);
  std::vector<int> fp32_store((size_t)n_layers, 0);
  // nodes whose value stays fp32 even in storage-rounding mode
  for (int i = 0; i < n_layers; ++i) {
    if (i == output_node || layers[i].op == ORC_SOFTMAX) fp32_store[(size_t)i] = 1;
    if (layers[i].op == ORC_FC) {
      bool any = false, all_softmax = true;
      for (int j = i + 1; j < n_layers; ++j)
        if (layers[j].input == i || layers[j].residual == i) {
          any = true;
          if (layers[j].op != ORC_SOFTMAX) all_softmax = false;
        }
      if (any && all_softmax) fp32_store[(size_t)i] = 1;
    }
  }
  for (int i = 0; i < n_layers; ++i) {
    const orc_layer& L = layers[i];
    if (L.input >= i || L.input < -1 || L.residual >= i) return -1;
    const float* in;
    int c, h, w;
    if (L.input == -1) { in = x; c = C; h = H; w = W; }
    else { const T& s = val[(size_t)L.input]; in = s.v.data(); c = s.c; h = s.h; w = s.w; }
    T& o = val[(size_t)i];
    switch (L.op) {
      case ORC_CONV: {
        if (L.cin != c) return -2;
        if (L.kw > 0 && L.kw != L.k) {   // rectangular kernel: padding only along the dimensions it extends over
          if (L.groups > 1) return -2;
          const int ph = L.k > 1 ? L.pad : 0, pw = L.kw > 1 ? L.pad : 0;
          o.c = L.cout; o.h = out_size(h, L.k, L.stride, ph); o.w = out_size(w, L.kw, L.stride, pw);
          o.v.resize((size_t)N * o.c * o.h * o.w);
          std::vector<float> wt = read_tensor(blob, L.w_off, (int64_t)L.cout * L.cin * L.k * L.kw, dtype);
          std::vector<float> bs = read_tensor(blob, L.b_off, L.cout, ORC_F32);
          orc_conv2d_rect(in, N, c, h, w, wt.data(), bs.data(), L.cout, L.k, L.kw, L.stride, ph, pw, o.v.data());
          break;
        }
        o.c = L.cout; o.h = out_size(h, L.k, L.stride, L.pad); o.w = out_size(w, L.k, L.stride, L.pad);
        o.v.resize((size_t)N * o.c * o.h * o.w);
        const int G = L.groups > 1 ? L.groups : 1;
        if (L.cin % G || L.cout % G) return -2;
        std::vector<float> wt = read_tensor(blob, L.w_off, (int64_t)L.cout * (L.cin / G) * L.k * L.k, dtype);
        std::vector<float> bs = read_tensor(blob, L.b_off, L.cout, ORC_F32);
        if (G == 1) orc_conv2d(in, N, c, h, w, wt.data(), bs.data(), L.cout, L.k, L.stride, L.pad, o.v.data());
        else orc_conv2d_grouped(in, N, c, h, w, wt.data(), bs.data(), L.cout, L.k, L.stride, L.pad, G, o.v.data());
        break;
      }
      case ORC_DWCONV: {
        if (L.cin != c || L.cout != c) return -2;
        o.c = c; o.h = out_size(h, L.k, L.stride, L.pad); o.w = out_size(w, L.k, L.stride, L.pad);
        o.v.resize((size_t)N * o.c * o.h * o.w);
        std::vector<float> wt = read_tensor(blob, L.w_off, (int64_t)c * L.k * L.k, dtype);
        std::vector<float> bs = read_tensor(blob, L.b_off, c, ORC_F32);
        orc_dwconv2d(in, N, c, h, w, wt.data(), bs.data(), L.k, L.stride, L.pad, o.v.data());
        break;
      }
      case ORC_MAXPOOL: {
        o.c = c;
        o.h = L.ceil_mode ? out_size_ceil(h, L.k, L.stride, L.pad) : out_size(h, L.k, L.stride, L.pad);
        o.w = L.ceil_mode ? out_size_ceil(w, L.k, L.stride, L.pad) : out_size(w, L.k, L.stride, L.pad);
        o.v.resize((size_t)N * o.c * o.h * o.w);
        orc_maxpool2d_ex(in, N, c, h, w, L.k, L.stride, L.pad, L.ceil_mode, o.v.data());
        break;
      }
      case ORC_MUL: {
        if (L.residual < 0) return -1;
        const T& gt = val[(size_t)L.residual];
        if (gt.c != c || gt.h != 1 || gt.w != 1) return -2;
        o.c = c; o.h = h; o.w = w;
        o.v.resize((size_t)N * c * h * w);
        orc_channel_scale(in, gt.v.data(), N, c, h, w, o.v.data());
        break;
      }
      case ORC_SLICE: {
        if (L.c_first < 0 || L.cout < 1 || L.c_first + L.cout > c) return -2;
        o.c = L.cout; o.h = h; o.w = w;
        o.v.resize((size_t)N * o.c * h * w);
        orc_slice(in, N, c, h, w, L.c_first, L.cout, o.v.data());
        break;
      }
      case ORC_SHUFFLE: {
        if (L.groups < 1 || c % L.groups) return -2;
        o.c = c; o.h = h; o.w = w;
        o.v.resize((size_t)N * c * h * w);
        orc_channel_shuffle(in, N, c, h, w, L.groups, o.v.data());
        break;
      }
      case ORC_AVGPOOL: {
        o.c = c; o.h = out_size(h, L.k, L.stride, L.pad); o.w = out_size(w, L.k, L.stride, L.pad);
        o.v.resize((size_t)N * o.c * o.h * o.w);
        orc_avgpool2d(in, N, c, h, w, L.k, L.stride, L.pad, o.v.data());
        break;
      }
      case ORC_CONCAT: {
        if (L.residual < 0) return -1;
        const T& s2 = val[(size_t)L.residual];
        if (s2.h != h || s2.w != w || L.cout != c + s2.c) return -2;
        o.c = c + s2.c; o.h = h; o.w = w;
        o.v.resize((size_t)N * o.c * o.h * o.w);
        orc_concat(in, c, s2.v.data(), s2.c, N, h, w, o.v.data());
        break;
      }
      case ORC_GAP: {
        o.c = c; o.h = 1; o.w = 1;
        o.v.resize((size_t)N * c);
        orc_global_avgpool(in, N, c, h, w, o.v.data());
        break;
      }
      case ORC_FC: {
        if (L.cin != c * h * w) return -2;
        o.c = L.cout; o.h = 1; o.w = 1;
        o.v.resize((size_t)N * L.cout);
        std::vector<float> wt = read_tensor(blob, L.w_off, (int64_t)L.cout * L.cin, dtype);
        std::vector<float> bs = read_tensor(blob, L.b_off, L.cout, ORC_F32);
        orc_fc(in, N, L.cin, wt.data(), bs.data(), L.cout, o.v.data());
        break;
      }
      case ORC_SOFTMAX: {
        if (h != 1 || w != 1) return -2;
        o.c = c; o.h = 1; o.w = 1;
        o.v.resize((size_t)N * c);
        orc_softmax(in, N, c, o.v.data());
        break;
      }
      default:
        return -1;
    }
    if (L.op == ORC_CONV || L.op == ORC_DWCONV || L.op == ORC_FC) {
      if (L.residual >= 0) {
        const T& s = val[(size_t)L.residual];
        if (s.c != o.c || s.h != o.h || s.w != o.w) return -2;
        orc_add(o.v.data(), s.v.data(), (int64_t)o.v.size());
      }
      orc_activate(o.v.data(), (int64_t)o.v.size(), L.act);
    }
    if (round_storage && !fp32_store[(size_t)i] && L.op != ORC_MAXPOOL)
      orc_round_bf16(o.v.data(), (int64_t)o.v.size());
  }
  const T& r = val[(size_t)return_node];
  if ((int64_t)r.v.size() > out_cap) return -3;
  std::memcpy(out, r.v.data(), r.v.size() * sizeof(float));
  return (int64_t)r.v.size();
}

int orc_acc_bytes(void) { return (int)sizeof(acc_t); }

}  // extern "C"
