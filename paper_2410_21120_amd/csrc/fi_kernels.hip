// HIP kernels of the fused DAG for gfx950 (wave64, MFMA).
//
// Every kernel is a GROUPED kernel: one launch carries 1..FI_MAX_GROUP independent
// problems (nodes of different member models at the same depth).  A workgroup finds its
// problem from the table of starting workgroup indices that travels with the launch's
// arguments; it then touches only that problem's input, weights and output, so a
// member's bits never depend on which other members share the launch (Section III-A,
// C1 and C4: no operator is merged across models, no tensor is shared between them).
//
// Tensors are NHWC with the channel stride padded to Cp; pad channels always hold zero.
// A tensor that the planner stored inside a concatenation's tensor has that tensor's pixel
// stride instead (Desc.xs / Desc.ys); a node the planner folded into its reader (a per-channel
// affine, a squeeze-excite scaling, a concatenation that a shuffle interleaves) has no launch.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "fi_device.h"
#include "fi_internal.h"

namespace fi {

// Workgroups a problem needs, as a function of the batch (host and device agree on this).
__host__ __device__ inline int problem_blocks(int kind, int tile, const Desc& d, int batch) {
  switch (kind) {
    case K_STAGE: return (batch * d.H * d.W + 255) / 256;
    case K_CONV_DIRECT: return (int)(((int64_t)batch * d.Ho * d.Wo * d.Cop + 255) / 256);
    case K_CONV_MFMA: {
      const int bm = tile_bm(tile);
      return ((batch * d.Ho * d.Wo + bm - 1) / bm) * d.tiles_n * d.splits;
    }
    case K_DWCONV: {
      const int strip = d.tiles_n > 1 ? d.tiles_n : 1;   // outputs per thread along a row (strip kernel)
      return (int)(((int64_t)batch * d.Ho * ((d.Wo + strip - 1) / strip) * (d.vec ? d.Cop / 8 : d.Cop) + 255) / 256);
    }
    case K_MAXPOOL:
    case K_AVGPOOL: {
      if (d.vec && d.tiles_n > 1) return (int)(((int64_t)batch * d.Ho * ((d.Wo + d.tiles_n - 1) / d.tiles_n) * (d.Cop / 8) + 255) / 256);   // strip kernel
      return (int)(((int64_t)batch * d.Ho * d.Wo * (d.vec ? d.Cop / 8 : d.Cop) + 255) / 256);
    }
    case K_GAP: return d.vec ? batch * ((d.Cop / 8 + 7) / 8) : (batch * d.Cop + 255) / 256;
    case K_SOFTMAX: return batch;
    case K_FC: return tile == 1 ? d.tiles_n * ((batch + 31) / 32)   // every slice of a tile in one workgroup (fc_block_kernel)
                                : (d.tiles_n * d.splits * ((batch + 31) / 32) + 3) / 4;
    case K_REDUCE: return (batch * d.Ho * d.Wo * (d.Cop / 4) + 255) / 256;
    case K_GATHER: return (int)(((int64_t)batch * d.Ho * d.Wo * (d.vec ? d.Cop / 8 : d.Cop) + 255) / 256);
    case K_CONCAT:
    case K_MUL: return (int)(((int64_t)batch * d.Ho * d.Wo * (d.vec ? d.Cop / 8 : d.Cop) + 255) / 256);
  }
  return 0;
}

__device__ __forceinline__ bool find_problem(const KArgs& a, int, int, int& p, int& bid) {
  return find_problem_at(a, (int)blockIdx.x, p, bid);
}

// ---------------------------------------------------------------------------------
// input staging: caller's [B,H,W,C] (weight dtype) -> [B,H,W,Cp] in the activation dtype
// ---------------------------------------------------------------------------------
template <typename TI, typename TA>
__global__ void __launch_bounds__(256) stage_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_STAGE, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t pix = (int64_t)bid * 256 + threadIdx.x;
  if (pix >= (int64_t)batch * d.H * d.W) return;
  const TI* x = static_cast<const TI*>(a.ext_in[p]) + pix * d.C;
  TA* y = reinterpret_cast<TA*>(a.abase + d.y_off) + pix * d.Cp;
  for (int c = 0; c < d.Cp; ++c) st(y + c, c < d.C ? ld(x + c) : 0.0f);
}

// ---------------------------------------------------------------------------------
// direct convolution / FC: one thread per output element.  Used by fp32 models and by
// bf16 members that keep fp32 activations.
// ---------------------------------------------------------------------------------
template <typename TW, typename TA>
__global__ void __launch_bounds__(256) conv_direct_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_CONV_DIRECT, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  const int64_t M = (int64_t)batch * d.Ho * d.Wo;
  if (idx >= M * d.Cop) return;
  const int o = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  float v = 0.0f;
  if (o < d.Co) {
    const int q = (int)(m % d.Wo);
    const int pp = (int)((m / d.Wo) % d.Ho);
    const int n = (int)(m / ((int64_t)d.Wo * d.Ho));
    const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
    const TW* w = reinterpret_cast<const TW*>(a.wbase + d.w_off) + (int64_t)o * d.Kp;
    float acc = 0.0f;
    for (int r = 0; r < d.k; ++r) {
      const int ih = pp * d.stride - d.pad + r;
      if (ih < 0 || ih >= d.H) continue;
      for (int s = 0; s < d.kw; ++s) {
        const int iw = q * d.stride - d.pad_w + s;
        if (iw < 0 || iw >= d.W) continue;
        const TA* xr = x + (((int64_t)n * d.H + ih) * d.W + iw) * d.Cp;
        const TW* wr = w + (r * d.kw + s) * d.Cp;
        for (int c = 0; c < d.C; ++c) acc += ld(xr + c) * ld(wr + c);
      }
    }
    v = acc + reinterpret_cast<const float*>(a.wbase + d.b_off)[o];
    if (d.r_off != kNone) v += ld(reinterpret_cast<const TA*>(a.abase + d.r_off) + m * d.Cop + o);
    v = activate(v, d.act);
  }
  if (d.ext) {
    if (o < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + o] = v;
  } else if (d.out_f32) {
    reinterpret_cast<float*>(a.abase + d.y_off)[m * d.Cop + o] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + o, v);
  }
}

// ---------------------------------------------------------------------------------
// implicit-GEMM convolution / FC on MFMA.
//   rows  m = (n, p, q) output pixels      M = batch*Ho*Wo
//   cols  o = output channel               N = Co
//   red.  kk = (r, s, c), c innermost      K = k*k*Cp, weight rows padded to Kp (x32)
// Per 64-element reduction tile every thread fetches 16-byte vectors of A (input patches,
// through a buffer resource whose out-of-range reads return zero: that is the padding, the
// rows past M and the reduction tail) and of B (weights) into registers one tile ahead of
// the multiply, parks them in LDS, and the 4 waves consume them with 32x32x16 bf16 MFMAs
// accumulating in fp32.  The epilogue transposes the accumulators through LDS (fp32) so that
// bias, residual, activation and the single round-to-nearest-even to bf16 run on 8
// consecutive channels per thread with 16-byte coalesced residual loads and output stores.
// Workgroups are renumbered so that each XCD (blockIdx % 8) owns one contiguous run of
// tiles: neighbouring tiles, which share input rows and a member's weights, meet in one L2.
// ---------------------------------------------------------------------------------
// Finishes four consecutive features [o, o + 4) of output row n from their complete fp32 sums: bias
// (and residual), activation, zero in the padded features, store.  p: the problem's slot in the launch.
template <typename TA>
__device__ __forceinline__ void finish_row4(const KArgs& a, const Desc& d, int p, int n, int o, float4 sum) {
  const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.wbase + d.b_off) + o);
  float v[4] = {sum.x + b.x, sum.y + b.y, sum.z + b.z, sum.w + b.w};
  if (d.r_off != kNone) {
    const TA* r = reinterpret_cast<const TA*>(a.abase + d.r_off) + (int64_t)n * d.Cop + o;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] += ld(r + t);
  }
  activate_n<4>(v, d.act);
#pragma unroll
  for (int t = 0; t < 4; ++t) v[t] = (o + t < d.Co) ? v[t] : 0.0f;
  if (d.ext) {
    float* y = static_cast<float*>(a.ext_out[p]) + (int64_t)n * d.Co + o;
#pragma unroll
    for (int t = 0; t < 4; ++t)
      if (o + t < d.Co) y[t] = v[t];
  } else if (sizeof(TA) == 4 || d.out_f32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.abase + d.y_off) + (int64_t)n * d.ys + o) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + (int64_t)n * d.ys + o) =
        make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
  }
}

// WIDE: the member keeps fp32 activations.  Each fp32 input is split on the fly into
// hi = bf16(x) and lo = bf16(x - hi) (two bf16 terms carry 16 mantissa bits), both halves are
// multiplied by the bf16 weights into the same fp32 accumulator, and outputs / residuals stay
// fp32: bf16 matrix-core throughput at fp32-grade activation accuracy.
// C4: the input has 4 stored channels (an RGB-like model input); an 8-element reduction vector
// then spans two neighbouring filter taps and is gathered with two half-width loads.
// GROUPED: a grouped convolution (packed as dense rows that are zero outside the row's group).  A column
// tile then needs only the input channels of the groups its output channels belong to: per filter tap the
// reduction walks channels [c_lo, c_hi) (whole 64-element tiles; the planner guarantees Cp % 64 == 0)
// instead of all Cp.  The skipped products are exact zeros, so the sums are the dense walk's.
// PRE: a pointwise convolution whose input goes through a per-channel affine stage first,
// x' = act(x * scale[c] + shift[c]) rounded to bf16 (the 1x1 depthwise node in front of it, which then has no
// launch of its own): applied to every input vector between its load and its LDS store, with the depthwise
// kernel's operations (product and sum rounded separately, one rounding to bf16).  The input may sit inside a
// concatenation's tensor, so its pixel stride is Desc.xs.
// PRE == 2: the input is scaled by a per-(image, channel) gate instead, x' = x * gate[n][c] rounded to bf16 (the
// scaling node that ends a squeeze-excite block; fp32 product, one rounding: the scaling kernel's operation).
// DEPTH: reduction tiles in flight in registers.  One (a tile's loads overlap the multiply of the tile before) is enough
// where several workgroups share a compute unit; a launch of few workgroups with a long reduction (one or two per
// compute unit, nothing else to hide a load behind) takes three, at the price of 64 registers.
template <int TILE, int BM, int BN, int WGM, int WGN, bool WIDE, bool C4 = false, bool GROUPED = false, int PRE = 0, int DEPTH = 1>
__global__ void __launch_bounds__(WGM * WGN * 64) conv_mfma_kernel(KArgs a) {
  static_assert(!GROUPED || (!WIDE && !C4), "the group walk exists for bf16 activations with 8-channel vectors");
  static_assert(DEPTH == 1 || (!WIDE && !C4 && !GROUPED && PRE == 0), "deeper prefetch exists for the plain bf16 convolution");
  static_assert(!PRE || (!C4 && !GROUPED && (!WIDE || PRE == 2)),
                "input-side stages exist for dense pointwise convolutions: the affine one on bf16 activations, the gate on either");
  constexpr int NT = WGM * WGN * 64;     // threads per workgroup
  constexpr int RPP = NT / 8;            // tile rows staged per pass (8 threads per 64-element row)
  constexpr int AE = WIDE ? 4 : 2;       // bytes per stored activation element
  constexpr int AV = WIDE ? 2 : 1;       // 16-byte loads per 8-element A vector
  constexpr int AT = WIDE ? 2 : 1;       // A tiles in LDS (hi, lo)
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // per-wave sub-tile
  constexpr int MI = WTM / 32, NI = WTN / 32;
  constexpr int AR = BM / RPP, BR = BN / RPP;  // 8-element vectors each thread stages per tile
  constexpr int STAGE = (AT * BM + BN) * LDS_STRIDE;   // bf16 elements per LDS buffer
  constexpr int SMEM = STAGE * 2;
  __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM];
  bf16_t* const As = reinterpret_cast<bf16_t*>(smem);   // [AT][BM][LDS_STRIDE] then B
  bf16_t* const Bs = As + AT * BM * LDS_STRIDE;

  // locate the problem and the tile (block-uniform)
  int p, bid;
  if (!find_problem_at(a, xcd_contiguous((int)blockIdx.x, (int)gridDim.x), p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int M = batch * d.Ho * d.Wo;
  // Outputs far larger than the last-level cache are streamed past it; smaller ones are left to the
  // cache, which absorbs the store burst of a launch whose workgroups all finish together.
  const bool stream_out = (int64_t)M * d.Cop * 2 > (int64_t)STREAM_OUT_BYTES;
  const int tiles_mn = ((M + BM - 1) / BM) * d.tiles_n;
  const int split = bid / tiles_mn;  // split-K: this workgroup reduces one slice of K into a partial tile
  bid -= split * tiles_mn;
  const int m0 = (bid / d.tiles_n) * BM;
  const int n0 = (bid % d.tiles_n) * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  const bf16_t* __restrict__ w = reinterpret_cast<const bf16_t*>(a.wbase + d.w_off);
  // bytes of the input this launch may touch: all pixels at their stride (PRE: the last pixel ends after its Cp channels)
  const int x_bytes = PRE ? (int)((((int64_t)batch * d.H * d.W - 1) * d.xs + d.Cp) * AE) : (int)((int64_t)batch * d.H * d.W * d.Cp * AE);
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.abase + d.x_off), 0, batch > 0 ? x_bytes : 0, 0x00020000);
  const bf16_t* const pre_w = PRE == 1 ? reinterpret_cast<const bf16_t*>(a.wbase + d.pw_off)
                            : PRE == 2 ? reinterpret_cast<const bf16_t*>(a.abase + d.pw_off) : nullptr;   // scale vector / gate tensor
  const float* const pre_b = PRE == 1 ? reinterpret_cast<const float*>(a.wbase + d.pb_off)
                           : (PRE == 2 && WIDE) ? reinterpret_cast<const float*>(a.abase + d.pw_off) : nullptr;   // shift vector / fp32 gate tensor

  // staging assignment: thread -> (row, 8-element k vector); 8 threads cover one 128-byte row
  const int srow = tid >> 3, kvec = (tid & 7) * 8;
  // Per row: the byte offset of its window origin (n, p*stride-pad, q*stride-pad, 0) and which
  // filter rows / columns land inside the image (bit r: row r valid; bit 16+s: column s valid).
  int a_row[AR], a_rc[AR];
  int a_gate[PRE == 2 ? AR : 1];   // PRE == 2: element offset of the row's image in the gate tensor
  const float inv_wo = 1.0f / (float)d.Wo, inv_ho = 1.0f / (float)d.Ho, inv_k = 1.0f / (float)d.kw;
  const bool pointwise = d.k == 1 && d.kw == 1 && d.stride == 1 && d.pad == 0 && d.pad_w == 0;  // output pixel m reads input pixel m: nothing to decode
#pragma unroll
  for (int i = 0; i < AR; ++i) {
    const int m = m0 + srow + RPP * i;
    const bool ok = m < M;
    if constexpr (PRE == 2) a_gate[i] = ((ok ? m : 0) / (d.H * d.W)) * d.Cp;
    if (pointwise) {
      a_row[i] = (ok ? m : 0) * (PRE ? d.xs : d.Cp) * AE;
      a_rc[i] = ok ? 0x10001 : 0;
      continue;
    }
    const int mm = ok ? m : 0;
    const int t = fast_div(mm, d.Wo, inv_wo);
    const int q = mm - t * d.Wo;
    const int n = fast_div(t, d.Ho, inv_ho);
    const int pp = t - n * d.Ho;
    const int ih0 = pp * d.stride - d.pad, iw0 = q * d.stride - d.pad_w;
    a_row[i] = ((n * d.H + ih0) * d.W + iw0) * d.Cp * AE;
    const int rc = (int)(taps_inside(ih0, d.k, d.H) | (taps_inside(iw0, d.kw, d.W) << 16));
    a_rc[i] = ok ? rc : 0;  // rows past M read as zero
  }
  // Weights through a buffer resource as well: a vector that must read as zero (the half tile that ends a row padded
  // to 32 elements, every vector of the fetch that follows the last tile) takes an out-of-range offset, so the fetch
  // needs no branch and sits in one basic block with the multiply it overlaps.
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(w), 0, (int)((int64_t)d.Co * d.Kp * 2), 0x00020000);
  int b_row[BR];
#pragma unroll
  for (int i = 0; i < BR; ++i) {
    int o = n0 + srow + RPP * i;
    o = o < d.Co ? o : d.Co - 1;  // clamped rows are computed and discarded
    b_row[i] = (o * d.Kp + kvec) * 2;
  }
  // this thread's reduction position (r, s, c) for the tile being fetched
  int c_lo = 0, c_hi = d.Cp;   // channels walked per filter tap
  if constexpr (GROUPED) {
    const int g0 = n0 / d.gout, g1 = (min(n0 + BN, d.Co) - 1) / d.gout;   // groups of this tile's output channels
    c_lo = (g0 * d.gin) / BK * BK;
    c_hi = min(d.Cp, ((g1 + 1) * d.gin + BK - 1) / BK * BK);
  }
  const int c_len = c_hi - c_lo;
  const int ntiles_all = GROUPED ? d.k * d.kw * (c_len / BK) : (d.Kp + BK - 1) / BK;
  const int per_split = (ntiles_all + d.splits - 1) / d.splits;
  const int kt0 = split * per_split;
  const int ntiles = min(ntiles_all, kt0 + per_split);  // this workgroup multiplies tiles [kt0, ntiles)
  int kr, ks, kc;
  if constexpr (GROUPED) {
    const int per_tap = c_len / BK;
    const int rs = kt0 / per_tap;
    kc = c_lo + (kt0 - rs * per_tap) * BK + kvec;
    kr = rs / d.kw;
    ks = rs - kr * d.kw;
  } else {
    const int k0 = kt0 * BK + kvec;
    const int rs = k0 / d.Cp;
    kc = k0 - rs * d.Cp;
    kr = rs / d.kw;
    ks = rs - kr * d.kw;
  }

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // DEPTH register stages feed one LDS buffer: fetch DEPTH tiles ahead, two barriers per tile.
  u32x4 av[DEPTH][AR][AV];
  uint4 bv[DEPTH][BR];
  uint4 pre_s[DEPTH];    // PRE == 1: scale (8 bf16) and shift (8 fp32) of this thread's channels in the tile being fetched
  float4 pre_t[DEPTH][2];
  uint4 pre_g[DEPTH][PRE == 2 ? AR : 1][AV];   // PRE == 2: the gate vectors of this thread's rows
  const bool b_tail = (d.Kp % BK) != 0;  // weight rows are padded to 32: the last tile may be half
  const bool one_wrap = c_len >= BK;     // (block-uniform)

#define FI_FETCH(KT, S, LIVE)                                                                     \
  {                                                                                               \
    /* a fetch past the last tile: the top bit puts every offset out of range (plain arithmetic, so no branch on it) */ \
    const uint32_t dead = (LIVE) ? 0u : OOB;                                                      \
    if constexpr (!C4) {                                                                          \
      const int tvar = ((kr * d.W + ks) * d.Cp + kc) * AE;                                        \
      _Pragma("unroll") for (int i = 0; i < AR; ++i) {                                            \
        const bool ok = ((a_rc[i] >> kr) & (a_rc[i] >> (16 + ks)) & 1) != 0;                       \
        const uint32_t off = (ok ? (uint32_t)(a_row[i] + tvar) : OOB) | dead;                     \
        _Pragma("unroll") for (int h = 0; h < AV; ++h)                                            \
            av[S][i][h] = __builtin_amdgcn_raw_buffer_load_b128(xres, off + 16 * h, 0, 0);        \
      }                                                                                           \
    } else {                                                                                      \
      const int tap0 = ((KT) * BK + kvec) >> 2; /* elements 0-3: tap0, elements 4-7: tap0 + 1 */  \
      int tr[2], tc[2], tv[2];                                                                    \
      _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                             \
        tr[h] = fast_div(tap0 + h, d.kw, inv_k);                                                   \
        tc[h] = tap0 + h - tr[h] * d.kw;                                                           \
        tv[h] = (tr[h] * d.W + tc[h]) * 4 * AE;                                                   \
      }                                                                                           \
      _Pragma("unroll") for (int i = 0; i < AR; ++i) {                                            \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                           \
          const bool ok = tr[h] < d.k && ((a_rc[i] >> tr[h]) & (a_rc[i] >> (16 + tc[h])) & 1) != 0; \
          const uint32_t off = (ok ? (uint32_t)(a_row[i] + tv[h]) : OOB) | dead;                  \
          if constexpr (WIDE) {                                                                   \
            av[S][i][h] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);                 \
          } else {                                                                                \
            const u32x2 half = __builtin_amdgcn_raw_buffer_load_b64(xres, off, 0, 0);             \
            av[S][i][0][2 * h] = half[0];                                                         \
            av[S][i][0][2 * h + 1] = half[1];                                                     \
          }                                                                                       \
        }                                                                                         \
      }                                                                                           \
    }                                                                                             \
    if constexpr (PRE == 2) {                                                                     \
      _Pragma("unroll") for (int i = 0; i < AR; ++i)                                              \
      _Pragma("unroll") for (int h = 0; h < AV; ++h) {                                            \
        if constexpr (WIDE) pre_g[S][i][h] = ((LIVE) && kr == 0) ? *reinterpret_cast<const uint4*>(pre_b + a_gate[i] + kc + 4 * h) : make_uint4(0, 0, 0, 0); \
        else pre_g[S][i][h] = ((LIVE) && kr == 0) ? *reinterpret_cast<const uint4*>(pre_w + a_gate[i] + kc) : make_uint4(0, 0, 0, 0); \
      }                                                                                           \
    }                                                                                             \
    if constexpr (PRE == 1) { /* channels past Cp (the tile tail) have walked on to filter row 1: no stage, the input reads as zero */ \
      const bool pok = (LIVE) && kr == 0;                                                                 \
      pre_s[S] = pok ? *reinterpret_cast<const uint4*>(pre_w + kc) : make_uint4(0, 0, 0, 0);      \
      pre_t[S][0] = pok ? *reinterpret_cast<const float4*>(pre_b + kc) : make_float4(0, 0, 0, 0); \
      pre_t[S][1] = pok ? *reinterpret_cast<const float4*>(pre_b + kc + 4) : make_float4(0, 0, 0, 0); \
    }                                                                                             \
    const bool bok = !(b_tail && (KT) == ntiles_all - 1 && kvec >= 32);                           \
    /* position of this tile in a weight row, in 8-element vectors past the thread's own kvec */  \
    const int wt = GROUPED ? ((kr * d.kw + ks) * d.Cp + kc - kvec) >> 3 : (KT) * (BK / 8);        \
    _Pragma("unroll") for (int i = 0; i < BR; ++i)                                                \
        bv[S][i] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wres, (bok ? (uint32_t)(b_row[i] + wt * 16) : OOB) | dead, 0, 0)); \
    kc += BK;                                                                                     \
    if (GROUPED || one_wrap) { /* at least 64 channels per tap: the walk leaves a tap at most once per tile */ \
      const bool wrap = kc >= c_hi;                                                               \
      kc -= wrap ? c_len : 0;                                                                     \
      ks += wrap ? 1 : 0;                                                                         \
      const bool wrap2 = ks == d.kw;                                                              \
      ks = wrap2 ? 0 : ks;                                                                        \
      kr += wrap2 ? 1 : 0;                                                                        \
    } else {                                                                                      \
      _Pragma("unroll") for (int t = 0; t < 8; ++t) {                                             \
        const bool wrap = kc >= c_hi;                                                             \
        kc -= wrap ? c_len : 0;                                                                   \
        ks += wrap ? 1 : 0;                                                                       \
        const bool wrap2 = ks == d.kw;                                                            \
        ks = wrap2 ? 0 : ks;                                                                      \
        kr += wrap2 ? 1 : 0;                                                                      \
      }                                                                                           \
    }                                                                                             \
  }

#define FI_PARK(S) /* register stage S into the LDS buffer */                                      \
  {                                                                                               \
    bf16_t* const Ap = As;                                                                        \
    bf16_t* const Bp = Bs;                                                                        \
    _Pragma("unroll") for (int i = 0; i < AR; ++i) {                                              \
      if constexpr (PRE == 2 && !WIDE) {                                                          \
        const uint32_t gw[4] = {pre_g[S][i][0].x, pre_g[S][i][0].y, pre_g[S][i][0].z, pre_g[S][i][0].w}; \
        u32x4 pk;                                                                                 \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                           \
          const uint32_t xw = av[S][i][0][e];                                                     \
          pk[e] = pack_bf16x2(__fmul_rn(__uint_as_float(xw << 16), __uint_as_float(gw[e] << 16)), \
                              __fmul_rn(__uint_as_float(xw & 0xFFFF0000u), __uint_as_float(gw[e] & 0xFFFF0000u))); \
        }                                                                                         \
        *reinterpret_cast<u32x4*>(&Ap[(srow + RPP * i) * LDS_STRIDE + kvec]) = pk;                \
      } else if constexpr (PRE == 1) {                                                            \
        const uint32_t sw[4] = {pre_s[S].x, pre_s[S].y, pre_s[S].z, pre_s[S].w};                  \
        const float sh[8] = {pre_t[S][0].x, pre_t[S][0].y, pre_t[S][0].z, pre_t[S][0].w,          \
                             pre_t[S][1].x, pre_t[S][1].y, pre_t[S][1].z, pre_t[S][1].w};         \
        float v[8];                                                                               \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                           \
          const uint32_t xw = av[S][i][0][e];                                                     \
          v[2 * e] = __fadd_rn(__fmul_rn(__uint_as_float(xw << 16), __uint_as_float(sw[e] << 16)), sh[2 * e]); \
          v[2 * e + 1] = __fadd_rn(__fmul_rn(__uint_as_float(xw & 0xFFFF0000u), __uint_as_float(sw[e] & 0xFFFF0000u)), sh[2 * e + 1]); \
        }                                                                                         \
        activate_n<8>(v, d.pre_act);                                                              \
        u32x4 pk;                                                                                 \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]); \
        *reinterpret_cast<u32x4*>(&Ap[(srow + RPP * i) * LDS_STRIDE + kvec]) = pk;                \
      } else if constexpr (!WIDE) {                                                               \
        *reinterpret_cast<u32x4*>(&Ap[(srow + RPP * i) * LDS_STRIDE + kvec]) = av[S][i][0];       \
      } else {                                                                                    \
        u32x4 hi, lo;                                                                             \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                           \
          float x0 = __uint_as_float(av[S][i][e >> 1][(2 * e) & 3]);                              \
          float x1 = __uint_as_float(av[S][i][e >> 1][(2 * e + 1) & 3]);                          \
          if constexpr (PRE == 2) { /* fp32 tensors: the scaled value is an fp32 product, as the scaling kernel stores it */ \
            const uint4 gq = pre_g[S][i][e >> 1];                                                 \
            const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};                                      \
            x0 = x0 * __uint_as_float(gw[(2 * e) & 3]);                                           \
            x1 = x1 * __uint_as_float(gw[(2 * e + 1) & 3]);                                       \
            /* the product is rounded to fp32 here, as the stored tensor would be: keep the compiler from */ \
            /* contracting it into the subtraction of the hi term below (an fma would skip that rounding) */ \
            asm volatile("" : "+v"(x0), "+v"(x1));                                                \
          }                                                                                       \
          const uint32_t h0 = f2bf(x0), h1 = f2bf(x1);                                            \
          hi[e] = h0 | (h1 << 16);                                                                \
          lo[e] = pack_bf16x2(x0 - __uint_as_float(h0 << 16), x1 - __uint_as_float(h1 << 16));    \
        }                                                                                         \
        *reinterpret_cast<u32x4*>(&Ap[(srow + RPP * i) * LDS_STRIDE + kvec]) = hi;                \
        *reinterpret_cast<u32x4*>(&Ap[(BM + srow + RPP * i) * LDS_STRIDE + kvec]) = lo;           \
      }                                                                                           \
    }                                                                                             \
    _Pragma("unroll") for (int i = 0; i < BR; ++i)                                                \
        *reinterpret_cast<uint4*>(&Bp[(srow + RPP * i) * LDS_STRIDE + kvec]) = bv[S][i];          \
  }

  // weights are the first MFMA operand: a lane then holds, for ONE pixel, runs of 4 consecutive channels
#define FI_MULTIPLY()                                                                             \
  {                                                                                               \
    const bf16_t* const Ap = As;                                                                  \
    const bf16_t* const Bp = Bs;                                                                  \
    _Pragma("unroll") for (int kk = 0; kk < BK; kk += 16) {                                       \
      bf16x8 af[AT][MI], bfr[NI];                                                                 \
      const int kof = kk + (lane >> 5) * 8;                                                       \
      _Pragma("unroll") for (int h = 0; h < AT; ++h)                                              \
      _Pragma("unroll") for (int i = 0; i < MI; ++i)                                              \
          af[h][i] = *reinterpret_cast<const bf16x8*>(                                            \
              &Ap[(h * BM + wm * WTM + i * 32 + (lane & 31)) * LDS_STRIDE + kof]);                \
      _Pragma("unroll") for (int j = 0; j < NI; ++j)                                              \
          bfr[j] = *reinterpret_cast<const bf16x8*>(&Bp[(wn * WTN + j * 32 + (lane & 31)) * LDS_STRIDE + kof]); \
      _Pragma("unroll") for (int h = AT - 1; h >= 0; --h) /* small (lo) terms first */            \
      _Pragma("unroll") for (int i = 0; i < MI; ++i)                                              \
      _Pragma("unroll") for (int j = 0; j < NI; ++j)                                              \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[h][i], acc[i][j], 0, 0, 0); \
    }                                                                                             \
  }

  if constexpr (DEPTH == 1) {
    FI_FETCH(kt0, 0, kt0 < ntiles)
    for (int kt = kt0; kt < ntiles; ++kt) {
      FI_PARK(0)
      __syncthreads();
      const bool more = kt + 1 < ntiles;
      FI_FETCH(kt + 1, 0, more)  // in flight while this tile is multiplied (after the last tile: nothing but out-of-range offsets)
      FI_MULTIPLY()
      __syncthreads();  // every wave is done with this tile before it is overwritten
    }
  } else {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) { FI_FETCH(kt0 + u, u, kt0 + u < ntiles) }
    for (int kt = kt0; kt < ntiles; kt += DEPTH) {
#pragma unroll
      for (int u = 0; u < DEPTH; ++u) {
        const int t = kt + u;
        if (t < ntiles) {   // (block-uniform)
          FI_PARK(u)
          __syncthreads();
          FI_FETCH(t + DEPTH, u, t + DEPTH < ntiles)   // DEPTH tiles ahead: in flight through DEPTH multiplies
          FI_MULTIPLY()
          __syncthreads();
        }
      }
    }
  }
#undef FI_FETCH
#undef FI_PARK
#undef FI_MULTIPLY

  // Two epilogues.  Long reductions (the 256-row tile) drain wave by wave without workgroup
  // barriers; streaming tiles go through one workgroup-wide fp32 tile so that a row of BN
  // channels leaves as one contiguous run (wider HBM bursts matter more there).
  // The common case has a path of its own, chosen once: bf16 output into the arena, every stored channel a real one,
  // no split, identity / ReLU / ReLU6.  Residual rows come in and output rows leave through buffer resources that end
  // with the tensor's last row, so a row past M or a column past Cop takes an out-of-range offset instead of a
  // branch, the activation is two instructions a value, and each block of rows is finished in one basic block (its
  // LDS reads, loads and stores issued in batches).  Everything else takes the general path below it.
  // (members with fp32-stored activations take it too: fp32 residual rows in, fp32 rows out, two 16-byte pieces per 8 channels)
  const bool fast = d.splits == 1 && !d.ext && (WIDE || !d.out_f32) && d.Co == d.Cop &&
                    ((int64_t)M + BM) * d.ys * AE < (1ll << 31) && ((int64_t)M + BM) * d.Cop * AE < (1ll << 31);
  const bool has_res = d.r_off != kNone;
  const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(a.abase + (fast && has_res ? d.r_off : 0)), 0, fast && has_res && M > 0 ? (int)((int64_t)M * d.Cop * AE) : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      a.abase + (fast ? d.y_off : 0), 0, fast && M > 0 ? (int)((((int64_t)M - 1) * d.ys + d.Cop) * AE) : 0, 0x00020000);
  // without a residual the loads return zero and the addend becomes -0.0, which leaves every value as it is
  uint32_t res_and = has_res ? 0xFFFFFFFFu : 0u, res_or = has_res ? 0u : 0x80008000u;
  asm volatile("" : "+v"(res_and), "+v"(res_or));   // (kept from being turned into a select per value)
  // bias + residual + activation + the one rounding for 8 consecutive channels of one row
#define FI_SUM_8(V0, V1, R, VA, VB)                                                               \
  {                                                                                               \
    (VA)[0] = (V0).x + bias8[0]; (VA)[1] = (V0).y + bias8[1]; (VA)[2] = (V0).z + bias8[2]; (VA)[3] = (V0).w + bias8[3]; \
    (VB)[0] = (V1).x + bias8[4]; (VB)[1] = (V1).y + bias8[5]; (VB)[2] = (V1).z + bias8[6]; (VB)[3] = (V1).w + bias8[7]; \
    if constexpr (WIDE) { /* fp32 residual; none reads as +0.0, as on the general path */          \
      _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                             \
        (VA)[t] += __uint_as_float((R)[0][t]);                                                    \
        (VB)[t] += __uint_as_float((R)[AV - 1][t]);                                               \
      }                                                                                           \
    } else {                                                                                      \
      const uint32_t r0 = ((R)[0][0] & res_and) | res_or, r1 = ((R)[0][1] & res_and) | res_or;    \
      const uint32_t r2 = ((R)[0][2] & res_and) | res_or, r3 = ((R)[0][3] & res_and) | res_or;    \
      (VA)[0] += __uint_as_float(r0 << 16); (VA)[1] += __uint_as_float(r0 & 0xFFFF0000u);         \
      (VA)[2] += __uint_as_float(r1 << 16); (VA)[3] += __uint_as_float(r1 & 0xFFFF0000u);         \
      (VB)[0] += __uint_as_float(r2 << 16); (VB)[1] += __uint_as_float(r2 & 0xFFFF0000u);         \
      (VB)[2] += __uint_as_float(r3 << 16); (VB)[3] += __uint_as_float(r3 & 0xFFFF0000u);         \
    }                                                                                             \
  }
#define FI_PACK_8(VA, VB, PK)                                                                     \
  {                                                                                               \
    if constexpr (WIDE) {                                                                         \
      _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                             \
        (PK)[0][t] = __float_as_uint((VA)[t]);                                                    \
        (PK)[AV - 1][t] = __float_as_uint((VB)[t]);                                               \
      }                                                                                           \
    } else {                                                                                      \
      (PK)[0][0] = pack_bf16x2((VA)[0], (VA)[1]); (PK)[0][1] = pack_bf16x2((VA)[2], (VA)[3]);     \
      (PK)[0][2] = pack_bf16x2((VB)[0], (VB)[1]); (PK)[0][3] = pack_bf16x2((VB)[2], (VB)[3]);     \
    }                                                                                             \
  }
  // a row's 8 channels: residual pieces in, finished pieces out (one 16-byte piece for bf16, two for fp32)
#define FI_LOAD_RES(RQ, ROW)                                                                      \
  _Pragma("unroll") for (int h = 0; h < AV; ++h)                                                  \
      (RQ)[h] = __builtin_amdgcn_raw_buffer_load_b128(rres, ((uint32_t)(((ROW) * d.Cop + o) * AE) + 16 * h) | col_dead, 0, 0);
#define FI_STORE_ROW(PK, ROW, AUX)                                                                \
  _Pragma("unroll") for (int h = 0; h < AV; ++h)                                                  \
      __builtin_amdgcn_raw_buffer_store_b128((PK)[h], yres, ((uint32_t)(((ROW) * d.ys + o) * AE) + 16 * h) | col_dead, 0, AUX);
  // The rows of one block: sums for every chunk, the activation (identity / ReLU / ReLU6 as two instructions a value;
  // a smooth one behind ONE branch for everything the thread holds of the block), the one rounding.  READ(ch, v0, v1)
  // fetches chunk ch of the block from the LDS tile.
#define FI_FINISH_BLOCK(RQ, PK, READ)                                                             \
  {                                                                                               \
    float vs[CH][8];                                                                              \
    _Pragma("unroll") for (int ch = 0; ch < CH; ++ch) {                                           \
      float4 v0, v1;                                                                              \
      READ(ch, v0, v1)                                                                            \
      float va[4], vb[4];                                                                         \
      FI_SUM_8(v0, v1, (RQ)[ch], va, vb)                                                          \
      if (!smooth) { clamp.apply(va); clamp.apply(vb); }                                          \
      _Pragma("unroll") for (int t = 0; t < 4; ++t) { vs[ch][t] = va[t]; vs[ch][4 + t] = vb[t]; } \
    }                                                                                             \
    if (smooth) activate_n<CH * 8>(&vs[0][0], d.act);                                             \
    _Pragma("unroll") for (int ch = 0; ch < CH; ++ch) {                                           \
      float va[4] = {vs[ch][0], vs[ch][1], vs[ch][2], vs[ch][3]}, vb[4] = {vs[ch][4], vs[ch][5], vs[ch][6], vs[ch][7]}; \
      FI_PACK_8(va, vb, (PK)[ch])                                                                 \
    }                                                                                             \
  }
  const bool smooth = d.act > FI_ACT_RELU6;
  if constexpr (BM == 256) {
    // ---- epilogue: every wave transposes its own sub-tile through a private LDS patch -----------
    // (no workgroup barrier: waves drain independently, one 32-row MFMA block at a time).  With the
    // weights as the first MFMA operand a lane holds, for pixel (lane & 31), four runs of 4
    // consecutive channels, parked with 16-byte LDS writes; it reads back 8 consecutive channels
    // of one row, so bias + residual + activation + the single rounding to bf16 work on 16-byte
    // vectors and every output row segment (WTN channels) is one contiguous store run.  The
    // block's residual vectors are requested before the accumulators are parked.
    constexpr int EPS = WTN + 4;                 // fp32 row stride of the patch (16-byte writes hit all banks)
    constexpr int CPR = WTN / 8;                 // 8-channel chunks per patch row
    constexpr int CH = 32 * CPR / 64;            // chunks per lane per 32-row block
    constexpr int RSTEP = 64 / CPR;              // row distance between a lane's chunks
    static_assert(4 * 32 * EPS * 4 <= SMEM, "epilogue patches fit in the tile memory");
    float* const ep = reinterpret_cast<float*>(smem) + wave * 32 * EPS;
    const int cc = (lane % CPR) * 8, lr0 = lane / CPR;
    const int o = n0 + wn * WTN + cc;
    const bool col_ok = o < d.Cop;
    float bias8[8];
    {
      const float* bias = reinterpret_cast<const float*>(a.wbase + d.b_off);
      const float4 b0 = col_ok ? *reinterpret_cast<const float4*>(bias + o) : make_float4(0, 0, 0, 0);
      const float4 b1 = col_ok ? *reinterpret_cast<const float4*>(bias + o + 4) : make_float4(0, 0, 0, 0);
      bias8[0] = b0.x; bias8[1] = b0.y; bias8[2] = b0.z; bias8[3] = b0.w;
      bias8[4] = b1.x; bias8[5] = b1.y; bias8[6] = b1.z; bias8[7] = b1.w;
    }
    const uint8_t* __restrict__ res = d.r_off != kNone ? a.abase + d.r_off : nullptr;
    if (fast) {
      const Activation<false> clamp(d.act);
      const uint32_t col_dead = col_ok ? 0u : OOB;
  #pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int mb = m0 + wm * WTM + i * 32;
        u32x4 rq[CH][AV], pk[CH][AV];
  #pragma unroll
        for (int ch = 0; ch < CH; ++ch) { FI_LOAD_RES(rq[ch], mb + lr0 + ch * RSTEP) }
  #pragma unroll
        for (int j = 0; j < NI; ++j)
  #pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<float4*>(&ep[(lane & 31) * EPS + j * 32 + 8 * g + 4 * (lane >> 5)]) =
                make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#define FI_READ_CHUNK(ch, v0, v1)                                                                 \
          v0 = *reinterpret_cast<const float4*>(&ep[(lr0 + (ch) * RSTEP) * EPS + cc]);            \
          v1 = *reinterpret_cast<const float4*>(&ep[(lr0 + (ch) * RSTEP) * EPS + cc + 4]);
        FI_FINISH_BLOCK(rq, pk, FI_READ_CHUNK)
#undef FI_READ_CHUNK
        if (stream_out) {
  #pragma unroll
          for (int ch = 0; ch < CH; ++ch) { FI_STORE_ROW(pk[ch], mb + lr0 + ch * RSTEP, 2) }
        } else {
  #pragma unroll
          for (int ch = 0; ch < CH; ++ch) { FI_STORE_ROW(pk[ch], mb + lr0 + ch * RSTEP, 0) }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      return;
    }
  #pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int mb = m0 + wm * WTM + i * 32;  // first output row of this MFMA block
      uint4 rv[CH][AV];
  #pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        const int m = mb + lr0 + ch * RSTEP;
  #pragma unroll
        for (int h = 0; h < AV; ++h) {
          rv[ch][h] = make_uint4(0, 0, 0, 0);
          if (res && d.splits == 1 && col_ok && m < M)
            rv[ch][h] = *reinterpret_cast<const uint4*>(res + ((int64_t)m * d.Cop + o) * AE + 16 * h);
        }
      }
  #pragma unroll
      for (int j = 0; j < NI; ++j)
  #pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(&ep[(lane & 31) * EPS + j * 32 + 8 * g + 4 * (lane >> 5)]) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the wave's own LDS writes precede its reads
  #pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        const int lr = lr0 + ch * RSTEP;
        const int m = mb + lr;
        float v[8];
        const float4 v0 = *reinterpret_cast<const float4*>(&ep[lr * EPS + cc]);
        const float4 v1 = *reinterpret_cast<const float4*>(&ep[lr * EPS + cc + 4]);
        if (m >= M || !col_ok) continue;
        if (d.splits > 1) {  // raw partial sums; the reduce launch finishes the node
          float* ws = reinterpret_cast<float*>(a.wsbase + d.ws_off) + ((int64_t)split * M + m) * d.Cop + o;
          *reinterpret_cast<float4*>(ws) = v0;
          *reinterpret_cast<float4*>(ws + 4) = v1;
          continue;
        }
        v[0] = v0.x + bias8[0]; v[1] = v0.y + bias8[1]; v[2] = v0.z + bias8[2]; v[3] = v0.w + bias8[3];
        v[4] = v1.x + bias8[4]; v[5] = v1.y + bias8[5]; v[6] = v1.z + bias8[6]; v[7] = v1.w + bias8[7];
        if constexpr (WIDE) {
          const uint4 r0 = rv[ch][0], r1 = rv[ch][AV - 1];
          v[0] += __uint_as_float(r0.x); v[1] += __uint_as_float(r0.y); v[2] += __uint_as_float(r0.z); v[3] += __uint_as_float(r0.w);
          v[4] += __uint_as_float(r1.x); v[5] += __uint_as_float(r1.y); v[6] += __uint_as_float(r1.z); v[7] += __uint_as_float(r1.w);
        } else {
          const uint4 r = rv[ch][0];
          v[0] += __uint_as_float(r.x << 16); v[1] += __uint_as_float(r.x & 0xFFFF0000u);
          v[2] += __uint_as_float(r.y << 16); v[3] += __uint_as_float(r.y & 0xFFFF0000u);
          v[4] += __uint_as_float(r.z << 16); v[5] += __uint_as_float(r.z & 0xFFFF0000u);
          v[6] += __uint_as_float(r.w << 16); v[7] += __uint_as_float(r.w & 0xFFFF0000u);
        }
        activate_n<8>(v, d.act);
  #pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = (o + t < d.Co) ? v[t] : 0.0f;  // pad channels hold zero
        if (d.ext) {
          float* y = static_cast<float*>(a.ext_out[p]) + (int64_t)m * d.Co + o;
  #pragma unroll
          for (int t = 0; t < 8; ++t)
            if (o + t < d.Co) y[t] = v[t];
        } else if (WIDE || d.out_f32) {
          float* y = reinterpret_cast<float*>(a.abase + d.y_off) + (int64_t)m * d.ys + o;
          *reinterpret_cast<float4*>(y) = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(y + 4) = make_float4(v[4], v[5], v[6], v[7]);
        } else {
            u32x4 pk;
          pk[0] = pack_bf16x2(v[0], v[1]); pk[1] = pack_bf16x2(v[2], v[3]);
          pk[2] = pack_bf16x2(v[4], v[5]); pk[3] = pack_bf16x2(v[6], v[7]);
          u32x4* const yp = reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + (int64_t)m * d.ys + o);
          if (stream_out) __builtin_nontemporal_store(pk, yp); else *yp = pk;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  // reads done before the next block's writes
    }
  } else {
    constexpr int EPS = BN + 4;                // fp32 row stride of the tile (16-byte writes spread over all banks)
    static_assert(64 * EPS * 4 <= SMEM, "epilogue tile fits in the tile memory");
    // ---- epilogue: 64 output rows per pass through an fp32 LDS tile ----------------------
    // A thread owns one 8-channel column chunk (the same in every pass) and CH rows per pass.
    // The pass's residual vectors are requested before the accumulators are parked, so their
    // latency overlaps the LDS round trip instead of serialising behind it.
    constexpr int CPR = BN / 8;          // 8-channel chunks per tile row
    constexpr int CH = 64 * CPR / NT;    // chunks per thread per pass
    constexpr int RSTEP = NT / CPR;      // row distance between a thread's chunks
    float* ep = reinterpret_cast<float*>(smem);
    const int cc = (tid % CPR) * 8, lr0 = tid / CPR;
    const int o = n0 + cc;
    const bool col_ok = o < d.Cop;
    float bias8[8];
    {
      const float* bias = reinterpret_cast<const float*>(a.wbase + d.b_off);
      const float4 b0 = col_ok ? *reinterpret_cast<const float4*>(bias + o) : make_float4(0, 0, 0, 0);
      const float4 b1 = col_ok ? *reinterpret_cast<const float4*>(bias + o + 4) : make_float4(0, 0, 0, 0);
      bias8[0] = b0.x; bias8[1] = b0.y; bias8[2] = b0.z; bias8[3] = b0.w;
      bias8[4] = b1.x; bias8[5] = b1.y; bias8[6] = b1.z; bias8[7] = b1.w;
    }
    const uint8_t* __restrict__ res = d.r_off != kNone ? a.abase + d.r_off : nullptr;
    if (fast) {
      const Activation<false> clamp(d.act);
      const uint32_t col_dead = col_ok ? 0u : OOB;
  #pragma unroll
      for (int pass = 0; pass < BM / 64; ++pass) {
        const int mp = m0 + pass * 64 + lr0;
        u32x4 rq[CH][AV], pk[CH][AV];
  #pragma unroll
        for (int ch = 0; ch < CH; ++ch) { FI_LOAD_RES(rq[ch], mp + ch * RSTEP) }
        if (pass > 0) __syncthreads();
  #pragma unroll
        for (int i = 0; i < MI; ++i) {
          const int rb = wm * WTM + i * 32;
          if (rb / 64 != pass) continue;
          const int lr = rb - pass * 64 + (lane & 31);
  #pragma unroll
          for (int j = 0; j < NI; ++j)
  #pragma unroll
            for (int g = 0; g < 4; ++g)
              *reinterpret_cast<float4*>(&ep[lr * EPS + wn * WTN + j * 32 + 8 * g + 4 * (lane >> 5)]) =
                  make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        }
        __syncthreads();
#define FI_READ_CHUNK(ch, v0, v1)                                                                 \
          v0 = *reinterpret_cast<const float4*>(&ep[(lr0 + (ch) * RSTEP) * EPS + cc]);            \
          v1 = *reinterpret_cast<const float4*>(&ep[(lr0 + (ch) * RSTEP) * EPS + cc + 4]);
        FI_FINISH_BLOCK(rq, pk, FI_READ_CHUNK)
#undef FI_READ_CHUNK
        if (stream_out) {
  #pragma unroll
          for (int ch = 0; ch < CH; ++ch) { FI_STORE_ROW(pk[ch], mp + ch * RSTEP, 2) }
        } else {
  #pragma unroll
          for (int ch = 0; ch < CH; ++ch) { FI_STORE_ROW(pk[ch], mp + ch * RSTEP, 0) }
        }
      }
      return;
    }
  #pragma unroll
    for (int pass = 0; pass < BM / 64; ++pass) {
      uint4 rv[CH][AV];
  #pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        const int m = m0 + pass * 64 + lr0 + ch * RSTEP;
  #pragma unroll
        for (int h = 0; h < AV; ++h) {
          rv[ch][h] = make_uint4(0, 0, 0, 0);
          if (res && d.splits == 1 && col_ok && m < M) rv[ch][h] = *reinterpret_cast<const uint4*>(res + ((int64_t)m * d.Cop + o) * AE + 16 * h);
        }
      }
      if (pass > 0) __syncthreads();
  #pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int rb = wm * WTM + i * 32;  // first row of this MFMA block inside the tile
        if (rb / 64 != pass) continue;
        // with the weights as the first MFMA operand a lane holds, for pixel (lane & 31), four runs
        // of 4 consecutive channels: 16-byte LDS writes
        const int lr = rb - pass * 64 + (lane & 31);
  #pragma unroll
        for (int j = 0; j < NI; ++j)
  #pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<float4*>(&ep[lr * EPS + wn * WTN + j * 32 + 8 * g + 4 * (lane >> 5)]) =
                make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      }
      __syncthreads();
  #pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        const int lr = lr0 + ch * RSTEP;
        const int m = m0 + pass * 64 + lr;
        if (m >= M || !col_ok) continue;
        float v[8];
        const float4 v0 = *reinterpret_cast<const float4*>(&ep[lr * EPS + cc]);
        const float4 v1 = *reinterpret_cast<const float4*>(&ep[lr * EPS + cc + 4]);
        if (d.splits > 1) {  // raw partial sums; the reduce launch finishes the node
          float* ws = reinterpret_cast<float*>(a.wsbase + d.ws_off) + ((int64_t)split * M + m) * d.Cop + o;
          *reinterpret_cast<float4*>(ws) = v0;
          *reinterpret_cast<float4*>(ws + 4) = v1;
          continue;
        }
        v[0] = v0.x + bias8[0]; v[1] = v0.y + bias8[1]; v[2] = v0.z + bias8[2]; v[3] = v0.w + bias8[3];
        v[4] = v1.x + bias8[4]; v[5] = v1.y + bias8[5]; v[6] = v1.z + bias8[6]; v[7] = v1.w + bias8[7];
        if constexpr (WIDE) {
          const uint4 r0 = rv[ch][0], r1 = rv[ch][AV - 1];
          v[0] += __uint_as_float(r0.x); v[1] += __uint_as_float(r0.y); v[2] += __uint_as_float(r0.z); v[3] += __uint_as_float(r0.w);
          v[4] += __uint_as_float(r1.x); v[5] += __uint_as_float(r1.y); v[6] += __uint_as_float(r1.z); v[7] += __uint_as_float(r1.w);
        } else {
          const uint4 r = rv[ch][0];
          v[0] += __uint_as_float(r.x << 16); v[1] += __uint_as_float(r.x & 0xFFFF0000u);
          v[2] += __uint_as_float(r.y << 16); v[3] += __uint_as_float(r.y & 0xFFFF0000u);
          v[4] += __uint_as_float(r.z << 16); v[5] += __uint_as_float(r.z & 0xFFFF0000u);
          v[6] += __uint_as_float(r.w << 16); v[7] += __uint_as_float(r.w & 0xFFFF0000u);
        }
        activate_n<8>(v, d.act);
  #pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (o + i < d.Co) ? v[i] : 0.0f;  // pad channels hold zero
        if (d.ext) {
          float* y = static_cast<float*>(a.ext_out[p]) + (int64_t)m * d.Co + o;
  #pragma unroll
          for (int i = 0; i < 8; ++i)
            if (o + i < d.Co) y[i] = v[i];
        } else if (WIDE || d.out_f32) {
          float* y = reinterpret_cast<float*>(a.abase + d.y_off) + (int64_t)m * d.ys + o;
          *reinterpret_cast<float4*>(y) = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(y + 4) = make_float4(v[4], v[5], v[6], v[7]);
        } else {
          uint4 pk;
          pk.x = pack_bf16x2(v[0], v[1]); pk.y = pack_bf16x2(v[2], v[3]);
          pk.z = pack_bf16x2(v[4], v[5]); pk.w = pack_bf16x2(v[6], v[7]);
            u32x4* const yp = reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + (int64_t)m * d.ys + o);
          if (stream_out) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, pk), yp); else *yp = __builtin_bit_cast(u32x4, pk);
        }
      }
    }
  }
#undef FI_SUM_8
#undef FI_PACK_8
#undef FI_LOAD_RES
#undef FI_STORE_ROW
#undef FI_FINISH_BLOCK
}

// ---------------------------------------------------------------------------------
// channel gather: output channel c is input channel pad + c (slice, stride == 0) or
// (c mod k) * (C / k) + c / k (shuffle in k groups, stride == 1), or channel c / 2 of the first (c even) or the second
// (c odd) of two sources of equal width (stride == 2: a concatenation shuffled in two groups, without building the
// concatenation; the second source sits at r_off with pixel stride tiles_n); values move unchanged
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) gather_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_GATHER, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  if (sizeof(TA) == 2 && d.vec) {   // bf16 tensors inside the arena: a thread gathers 8 output channels and stores them as one vector
    const int cv = d.Cop / 8;
    if (idx >= (int64_t)batch * d.Ho * d.Wo * cv) return;
    const int c8 = (int)(idx % cv) * 8;
    const int64_t m = idx / cv;
    const uint16_t* x = reinterpret_cast<const uint16_t*>(a.abase + d.x_off) + m * d.Cp;
    uint16_t* y = reinterpret_cast<uint16_t*>(a.abase + d.y_off) + m * d.ys + c8;
    if (d.stride == 0 && (d.pad & 7) == 0 && c8 + 8 <= d.Co) {   // aligned slice: the 8 channels are one vector of the source too
      *reinterpret_cast<uint4*>(y) = *reinterpret_cast<const uint4*>(x + d.pad + c8);
      return;
    }
    if (d.stride == 2) {   // interleave: four channels of each source make the eight outputs
      const uint16_t* xb = reinterpret_cast<const uint16_t*>(a.abase + d.r_off) + m * d.tiles_n;
      uint32_t w[4];
      if (c8 + 8 <= d.Co) {
        const uint2 va = *reinterpret_cast<const uint2*>(x + c8 / 2), vb = *reinterpret_cast<const uint2*>(xb + c8 / 2);
        w[0] = (va.x & 0xFFFFu) | (vb.x << 16); w[1] = (va.x >> 16) | (vb.x & 0xFFFF0000u);
        w[2] = (va.y & 0xFFFFu) | (vb.y << 16); w[3] = (va.y >> 16) | (vb.y & 0xFFFF0000u);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int c = c8 + i;
          const uint32_t v = c < d.Co ? ((c & 1) ? xb[c >> 1] : x[c >> 1]) : 0u;
          w[i >> 1] = (i & 1) ? (w[i >> 1] | (v << 16)) : v;
        }
      }
      *reinterpret_cast<uint4*>(y) = make_uint4(w[0], w[1], w[2], w[3]);
      return;
    }
    const int per = d.stride == 0 ? 0 : d.C / d.k;
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = c8 + i;
      const int src = d.stride == 0 ? d.pad + c : (c % d.k) * per + c / d.k;
      const uint32_t v = c < d.Co ? x[src] : 0u;   // values move as bits; channels past Co are zero padding
      w[i >> 1] = (i & 1) ? (w[i >> 1] | (v << 16)) : v;
    }
    *reinterpret_cast<uint4*>(y) = make_uint4(w[0], w[1], w[2], w[3]);
    return;
  }
  if (idx >= (int64_t)batch * d.Ho * d.Wo * d.Cop) return;
  const int c = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
  float v = 0.0f;
  if (c < d.Co) {
    const int src = d.stride == 0 ? d.pad + c : (c % d.k) * (d.C / d.k) + c / d.k;
    v = d.stride == 2 ? ((c & 1) ? ld(reinterpret_cast<const TA*>(a.abase + d.r_off) + m * d.tiles_n + (c >> 1)) : ld(x + m * d.Cp + (c >> 1)))
                      : ld(x + m * d.Cp + src);
  }
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + c] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + c, v);
  }
}

// ---------------------------------------------------------------------------------
// channel concatenation: output pixel = C channels of the first source (stride Cp), then Kp
// channels of the second (stride tiles_n), then zero padding up to Cop
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) concat_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_CONCAT, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  const TA* xa = reinterpret_cast<const TA*>(a.abase + d.x_off);
  const TA* xb = reinterpret_cast<const TA*>(a.abase + d.r_off);
  const int64_t M = (int64_t)batch * d.Ho * d.Wo;
  if (sizeof(TA) == 2 && d.vec) {  // C % 8 == 0: an 8-channel vector never straddles the two sources
    const int cv = d.Cop / 8;
    if (idx >= M * cv) return;
    const int c8 = (int)(idx % cv) * 8;
    const int64_t m = idx / cv;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (c8 < d.C) v = *reinterpret_cast<const uint4*>(xa + m * d.Cp + c8);
    else if (c8 - d.C < d.tiles_n) v = *reinterpret_cast<const uint4*>(xb + m * d.tiles_n + (c8 - d.C));  // the source's own pad channels are zero
    *reinterpret_cast<uint4*>(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + c8) = v;
    return;
  }
  if (idx >= M * d.Cop) return;
  const int c = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  float v = 0.0f;
  if (c < d.C) v = ld(xa + m * d.Cp + c);
  else if (c - d.C < d.Kp) v = ld(xb + m * d.tiles_n + (c - d.C));
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + c] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + c, v);
  }
}

// ---------------------------------------------------------------------------------
// depthwise convolution: one thread per (pixel, channel), channel fastest (coalesced)
// ---------------------------------------------------------------------------------
template <typename TW, typename TA>
__global__ void __launch_bounds__(256) dwconv_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_DWCONV, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  if (idx >= (int64_t)batch * d.Ho * d.Wo * d.Cop) return;
  const int c = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  const int q = (int)(m % d.Wo);
  const int pp = (int)((m / d.Wo) % d.Ho);
  const int n = (int)(m / ((int64_t)d.Wo * d.Ho));
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
  const TW* w = reinterpret_cast<const TW*>(a.wbase + d.w_off);
  float acc = 0.0f;
  for (int r = 0; r < d.k; ++r) {
    const int ih = pp * d.stride - d.pad + r;
    if (ih < 0 || ih >= d.H) continue;
    for (int s = 0; s < d.k; ++s) {
      const int iw = q * d.stride - d.pad + s;
      if (iw < 0 || iw >= d.W) continue;
      acc += ld(x + (((int64_t)n * d.H + ih) * d.W + iw) * d.Cp + c) * ld(w + (r * d.k + s) * d.Cp + c);
    }
  }
  float v = 0.0f;
  if (c < d.Co) {
    v = acc + reinterpret_cast<const float*>(a.wbase + d.b_off)[c];
    if (d.r_off != kNone) v += ld(reinterpret_cast<const TA*>(a.abase + d.r_off) + idx);
    v = activate(v, d.act);
  }
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + c] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + idx, v);
  }
}

// ---------------------------------------------------------------------------------
// window pooling: out-of-range taps are skipped.  Max: padding behaves as -inf and the result is
// one of the inputs (exact).  AVG: the in-range taps are summed in fp32 and divided by the full
// window area k*k (padding counts as zeros), rounded once on store.  One thread per (pixel,
// 8 channels) with 16-byte loads and stores when the channel stride allows it (bf16,
// Cp % 8 == 0); one thread per element otherwise.
// ---------------------------------------------------------------------------------
template <typename TA, bool AVG>
__global__ void __launch_bounds__(256) pool_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, AVG ? K_AVGPOOL : K_MAXPOOL, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
  if (sizeof(TA) == 2 && d.vec) {
    const int cv = d.Cp / 8;
    if (idx >= (int64_t)batch * d.Ho * d.Wo * cv) return;
    const int c8 = (int)(idx % cv) * 8;
    const int64_t m = idx / cv;
    const int q = (int)(m % d.Wo);
    const int pp = (int)((m / d.Wo) % d.Ho);
    const int n = (int)(m / ((int64_t)d.Wo * d.Ho));
    float best[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) best[i] = AVG ? 0.0f : -INFINITY;
    for (int r = 0; r < d.k; ++r) {
      const int ih = pp * d.stride - d.pad + r;
      if (ih < 0 || ih >= d.H) continue;
      for (int s = 0; s < d.k; ++s) {
        const int iw = q * d.stride - d.pad + s;
        if (iw < 0 || iw >= d.W) continue;
        const uint4 v = *reinterpret_cast<const uint4*>(x + (((int64_t)n * d.H + ih) * d.W + iw) * d.Cp + c8);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lo = __uint_as_float(u[i] << 16), hi = __uint_as_float(u[i] & 0xFFFF0000u);
          best[2 * i] = AVG ? best[2 * i] + lo : fmaxf(best[2 * i], lo);
          best[2 * i + 1] = AVG ? best[2 * i + 1] + hi : fmaxf(best[2 * i + 1], hi);
        }
      }
    }
    uint4 o;
    if constexpr (AVG) {
      const float area = (float)(d.k * d.k);
      o.x = pack_bf16x2(best[0] / area, best[1] / area); o.y = pack_bf16x2(best[2] / area, best[3] / area);
      o.z = pack_bf16x2(best[4] / area, best[5] / area); o.w = pack_bf16x2(best[6] / area, best[7] / area);
      *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + m * d.ys + c8) = o;
      return;
    }
    // the maxima are bf16 values already: packing is exact
    o.x = (__float_as_uint(best[0]) >> 16) | (__float_as_uint(best[1]) & 0xFFFF0000u);
    o.y = (__float_as_uint(best[2]) >> 16) | (__float_as_uint(best[3]) & 0xFFFF0000u);
    o.z = (__float_as_uint(best[4]) >> 16) | (__float_as_uint(best[5]) & 0xFFFF0000u);
    o.w = (__float_as_uint(best[6]) >> 16) | (__float_as_uint(best[7]) & 0xFFFF0000u);
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + m * d.ys + c8) = o;
    return;
  }
  if (idx >= (int64_t)batch * d.Ho * d.Wo * d.Cop) return;
  const int c = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  const int q = (int)(m % d.Wo);
  const int pp = (int)((m / d.Wo) % d.Ho);
  const int n = (int)(m / ((int64_t)d.Wo * d.Ho));
  float best = AVG ? 0.0f : -INFINITY;
  for (int r = 0; r < d.k; ++r) {
    const int ih = pp * d.stride - d.pad + r;
    if (ih < 0 || ih >= d.H) continue;
    for (int s = 0; s < d.k; ++s) {
      const int iw = q * d.stride - d.pad + s;
      if (iw < 0 || iw >= d.W) continue;
      const float v = ld(x + (((int64_t)n * d.H + ih) * d.W + iw) * d.Cp + c);
      best = AVG ? best + v : fmaxf(best, v);
    }
  }
  if (AVG) best = best / (float)(d.k * d.k);
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + c] = best;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + idx, best);
  }
}

// ---------------------------------------------------------------------------------
// 3x3 stride-1 window pooling in strip form (bf16 tensors, 8-channel vectors): a thread owns 4 neighbouring
// outputs of one output row.  Per window row it loads the 6 input pixels the strip touches once and feeds
// every output from them (18 loads for 4 outputs instead of 36); taps outside the image are skipped exactly
// as in pool_kernel, and every output combines its taps in the same (row, column) order.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void load8(const bf16_t* p, float* v);
__device__ __forceinline__ void store8(bf16_t* p, const float* v);
template <bool AVG>
__global__ void __launch_bounds__(256) pool_strip_kernel(KArgs a) {
  constexpr int S = 4, KS = 3, NPIX = S + KS - 1;
  int p, bid;
  if (!find_problem(a, AVG ? K_AVGPOOL : K_MAXPOOL, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int cv = d.Cp / 8, strips = (d.Wo + S - 1) / S;
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  if (idx >= (int64_t)batch * d.Ho * strips * cv) return;
  const int c8 = (int)(idx % cv) * 8;
  const int64_t t = idx / cv;
  const int q0 = (int)(t % strips) * S;
  const int pp = (int)((t / strips) % d.Ho);
  const int n = (int)(t / ((int64_t)strips * d.Ho));
  const bf16_t* const xn = reinterpret_cast<const bf16_t*>(a.abase + d.x_off) + (int64_t)n * d.H * d.W * d.Cp + c8;
  float best[S][8];
#pragma unroll
  for (int j = 0; j < S; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) best[j][i] = AVG ? 0.0f : -INFINITY;
  const int ih0 = pp - d.pad, iw0 = q0 - d.pad;
#pragma unroll
  for (int r = 0; r < KS; ++r) {
    const int ih = ih0 + r;
    if ((unsigned)ih >= (unsigned)d.H) continue;
    const bf16_t* const xr = xn + (int64_t)ih * d.W * d.Cp;
    float xv[NPIX][8];
    bool ok[NPIX];
#pragma unroll
    for (int c = 0; c < NPIX; ++c) {
      const int iw = iw0 + c;
      ok[c] = (unsigned)iw < (unsigned)d.W;
      load8(xr + (ok[c] ? (int64_t)iw * d.Cp : 0), xv[c]);   // always a valid address; skipped below when outside
    }
#pragma unroll
    for (int j = 0; j < S; ++j)
#pragma unroll
      for (int sx = 0; sx < KS; ++sx)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float v = xv[j + sx][i];
          best[j][i] = !ok[j + sx] ? best[j][i] : AVG ? best[j][i] + v : fmaxf(best[j][i], v);
        }
  }
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int q = q0 + j;
    if (q >= d.Wo) break;
    const int64_t m = ((int64_t)n * d.Ho + pp) * d.Wo + q;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = AVG ? best[j][i] / (float)(KS * KS) : best[j][i];
    store8(reinterpret_cast<bf16_t*>(a.abase + d.y_off) + m * d.ys + c8, v);   // maxima are bf16 values already: the rounding is exact
  }
}

// ---------------------------------------------------------------------------------
// global average pooling: one thread per (image, channel), fp32 sum, divide by H*W
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) gap_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_GAP, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int idx = bid * 256 + threadIdx.x;
  if (idx >= batch * d.Cop) return;
  const int c = idx % d.Cop, n = idx / d.Cop;
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off) + (int64_t)n * d.H * d.W * d.Cp + c;
  float sum = 0.0f;
  for (int i = 0; i < d.H * d.W; ++i) sum += ld(x + (int64_t)i * d.Cp);
  const float v = sum / (float)(d.H * d.W);
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[(int64_t)n * d.Co + c] = v;
  } else if (d.out_f32) {
    reinterpret_cast<float*>(a.abase + d.y_off)[idx] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + idx, v);
  }
}

// ---------------------------------------------------------------------------------
// softmax over the class axis of an fp32 [batch, Cp] tensor: one wave per row
// ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) softmax_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_SOFTMAX, 0, p, bid)) return;
  const Desc d = a.d[p];
  const float* z = reinterpret_cast<const float*>(a.abase + d.x_off) + (int64_t)bid * d.Cp;
  float* y = d.ext ? static_cast<float*>(a.ext_out[p]) + (int64_t)bid * d.Co
                   : reinterpret_cast<float*>(a.abase + d.y_off) + (int64_t)bid * d.Cop;
  const int lane = threadIdx.x;
  float m = -INFINITY;
  for (int c = lane; c < d.C; c += 64) m = fmaxf(m, z[c]);
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  float sum = 0.0f;
  for (int c = lane; c < d.C; c += 64) sum += expf(z[c] - m);
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
  for (int c = lane; c < d.C; c += 64) y[c] = expf(z[c] - m) / sum;
  if (!d.ext)
    for (int c = d.C + lane; c < d.Cop; c += 64) y[c] = 0.0f;
}

// ---------------------------------------------------------------------------------
// 8-channel vector access for the bandwidth-bound kernels
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void load8(const bf16_t* p, float* v) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xFFFF0000u);
  v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xFFFF0000u);
  v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xFFFF0000u);
  v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xFFFF0000u);
}
__device__ __forceinline__ void load8(const float* p, float* v) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void store8(bf16_t* p, const float* v) {
  uint4 u;
  u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]); u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = u;
}
__device__ __forceinline__ void store8(float* p, const float* v) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

// ---------------------------------------------------------------------------------
// per-(image, channel) gate: y[n,h,w,c] = x[n,h,w,c] * g[n,c], fp32 product, one rounding on store
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) mul_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_MUL, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
  const TA* g = reinterpret_cast<const TA*>(a.abase + d.r_off);
  const int64_t HW = (int64_t)d.Ho * d.Wo;
  if (sizeof(TA) == 2 && d.vec) {
    const int cv = d.Cop / 8;
    if (idx >= (int64_t)batch * HW * cv) return;
    const int c8 = (int)(idx % cv) * 8;
    const int64_t m = idx / cv;
    float xv[8], gv[8];
    load8(x + m * d.Cp + c8, xv);
    load8(g + (m / HW) * d.Cp + c8, gv);
#pragma unroll
    for (int i = 0; i < 8; ++i) xv[i] *= gv[i];
    store8(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + c8, xv);
    return;
  }
  if (idx >= (int64_t)batch * HW * d.Cop) return;
  const int c = (int)(idx % d.Cop);
  const int64_t m = idx / d.Cop;
  const float v = c < d.Co ? ld(x + m * d.Cp + c) * ld(g + (m / HW) * d.Cp + c) : 0.0f;
  if (d.ext) {
    if (c < d.Co) static_cast<float*>(a.ext_out[p])[m * d.Co + c] = v;
  } else {
    st(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.Cop + c, v);
  }
}


// ---------------------------------------------------------------------------------
// depthwise convolution, bf16 weights: one thread per (pixel, 8 channels); 16-byte (bf16) or
// 2x16-byte (fp32) activation vectors, coalesced along the channel axis.
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) dwconv_vec_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_DWCONV, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int cv = d.Cop / 8;
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  if (idx >= (int64_t)batch * d.Ho * d.Wo * cv) return;
  const int c8 = (int)(idx % cv) * 8;
  const int64_t m = idx / cv;
  const int q = (int)(m % d.Wo);
  const int pp = (int)((m / d.Wo) % d.Ho);
  const int n = (int)(m / ((int64_t)d.Wo * d.Ho));
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off);
  const bf16_t* w = reinterpret_cast<const bf16_t*>(a.wbase + d.w_off);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
  for (int r = 0; r < d.k; ++r) {
    const int ih = pp * d.stride - d.pad + r;
    if (ih < 0 || ih >= d.H) continue;
    for (int s = 0; s < d.k; ++s) {
      const int iw = q * d.stride - d.pad + s;
      if (iw < 0 || iw >= d.W) continue;
      float xv[8], wv[8];
      load8(x + (((int64_t)n * d.H + ih) * d.W + iw) * d.xs + c8, xv);
      load8(w + (r * d.k + s) * d.Cp + c8, wv);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += xv[i] * wv[i];
    }
  }
  float bv[8];
  load8(reinterpret_cast<const float*>(a.wbase + d.b_off) + c8, bv);
  if (d.r_off != kNone) {
    float rv[8];
    load8(reinterpret_cast<const TA*>(a.abase + d.r_off) + m * d.Cop + c8, rv);
#pragma unroll
    for (int i = 0; i < 8; ++i) bv[i] += rv[i];
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] += bv[i];
  activate_n<8>(acc, d.act);
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (c8 + i < d.Co) ? acc[i] : 0.0f;
  if (d.ext) {
    float* y = static_cast<float*>(a.ext_out[p]) + m * d.Co + c8;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (c8 + i < d.Co) y[i] = acc[i];
  } else {
    store8(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.ys + c8, acc);
  }
}

// ---------------------------------------------------------------------------------
// depthwise convolution, strip form (3x3 / 5x5 / 7x7, stride 1 or 2, 8-channel vectors): a thread owns
// S neighbouring outputs of one output row (S = 4 at stride 1, 2 at stride 2) for 8 channels.  Per filter
// row it loads the (S-1)*stride + KS input pixels the strip touches and the KS weight vectors once, and
// feeds every output from them: a third of the loads, address arithmetic and weight conversions of the
// one-output-per-thread form.  Each output still accumulates its taps in (r, s) order.
// ---------------------------------------------------------------------------------
template <typename TA, int KS, int ST>
__global__ void __launch_bounds__(256) dwconv_strip_kernel(KArgs a) {
  constexpr int S = ST == 1 ? 4 : 2;
  constexpr int NPIX = (S - 1) * ST + KS;
  int p, bid;
  if (!find_problem(a, K_DWCONV, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int cv = d.Cop / 8, strips = (d.Wo + S - 1) / S;
  const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
  if (idx >= (int64_t)batch * d.Ho * strips * cv) return;
  const int c8 = (int)(idx % cv) * 8;
  const int64_t t = idx / cv;
  const int q0 = (int)(t % strips) * S;
  const int pp = (int)((t / strips) % d.Ho);
  const int n = (int)(t / ((int64_t)strips * d.Ho));
  const TA* const xn = reinterpret_cast<const TA*>(a.abase + d.x_off) + (int64_t)n * d.H * d.W * d.xs + c8;
  const bf16_t* const w = reinterpret_cast<const bf16_t*>(a.wbase + d.w_off) + c8;
  float acc[S][8];
#pragma unroll
  for (int j = 0; j < S; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[j][i] = 0.0f;
  const int ih0 = pp * ST - d.pad, iw0 = q0 * ST - d.pad;
#pragma unroll
  for (int r = 0; r < KS; ++r) {
    const int ih = ih0 + r;
    if ((unsigned)ih >= (unsigned)d.H) continue;   // a row outside the image adds nothing
    const TA* const xr = xn + (int64_t)ih * d.W * d.xs;
    float xv[NPIX][8], wv[KS][8];
#pragma unroll
    for (int c = 0; c < NPIX; ++c) {
      const int iw = iw0 + c;
      const bool ok = (unsigned)iw < (unsigned)d.W;
      load8(xr + (ok ? (int64_t)iw * d.xs : 0), xv[c]);   // always a valid address; masked below
#pragma unroll
      for (int i = 0; i < 8; ++i) xv[c][i] = ok ? xv[c][i] : 0.0f;
    }
#pragma unroll
    for (int sx = 0; sx < KS; ++sx) load8(w + (r * KS + sx) * d.Cp, wv[sx]);
#pragma unroll
    for (int j = 0; j < S; ++j)
#pragma unroll
      for (int sx = 0; sx < KS; ++sx)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[j][i] += xv[j * ST + sx][i] * wv[sx][i];
  }
  float bv[8];
  load8(reinterpret_cast<const float*>(a.wbase + d.b_off) + c8, bv);
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int q = q0 + j;
    if (q >= d.Wo) break;
    const int64_t m = ((int64_t)n * d.Ho + pp) * d.Wo + q;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = acc[j][i] + bv[i];
    if (d.r_off != kNone) {
      float rv[8];
      load8(reinterpret_cast<const TA*>(a.abase + d.r_off) + m * d.Cop + c8, rv);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += rv[i];
    }
    activate_n<8>(v, d.act);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (c8 + i < d.Co) ? v[i] : 0.0f;
    if (d.ext) {
      float* y = static_cast<float*>(a.ext_out[p]) + m * d.Co + c8;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (c8 + i < d.Co) y[i] = v[i];
    } else {
      store8(reinterpret_cast<TA*>(a.abase + d.y_off) + m * d.ys + c8, v);
    }
  }
}

// ---------------------------------------------------------------------------------
// global average pooling, 8 channels per thread
// ---------------------------------------------------------------------------------
template <typename TA>
__global__ void __launch_bounds__(256) gap_vec_kernel(KArgs a) {
  // One workgroup = one image x 8 channel groups (128 contiguous bytes of a bf16 pixel) x 32 pixel phases:
  // thread (phase, group) sums pixels phase, phase + 32, ... of its 8 channels; the 8 phases of a wave are
  // added pairwise across lanes, the 4 waves' sums through LDS in wave order (a fixed tree: the order depends
  // on nothing but H*W).  A per-thread walk over all H*W pixels is one long chain of load latencies; this
  // keeps 32 pixels x 128 bytes in flight per workgroup.
  __shared__ float part[4][8][8];   // [wave][group][channel]
  int p, bid;
  if (!find_problem(a, K_GAP, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int cv = d.Cop / 8, cvb = (cv + 7) / 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = bid / cvb, gl = lane & 7, cg = (bid % cvb) * 8 + gl, phase = wave * 8 + (lane >> 3);
  const bool live = cg < cv;
  const int c8 = cg * 8;
  const int HW = d.H * d.W;
  const TA* x = reinterpret_cast<const TA*>(a.abase + d.x_off) + (int64_t)n * HW * d.Cp + c8;
  float sum[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) sum[i] = 0.0f;
  if (live)
    for (int t = phase; t < HW; t += 32) {
      float v[8];
      load8(x + (int64_t)t * d.Cp, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) sum[i] += v[i];
    }
#pragma unroll
  for (int step = 8; step < 64; step <<= 1)
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[i] += __shfl_xor(sum[i], step);
  if (lane < 8)
#pragma unroll
    for (int i = 0; i < 8; ++i) part[wave][gl][i] = sum[i];
  __syncthreads();
  if (wave != 0 || lane >= 8 || !live) return;
  const float hw = (float)HW;
#pragma unroll
  for (int i = 0; i < 8; ++i) sum[i] = (((part[0][gl][i] + part[1][gl][i]) + part[2][gl][i]) + part[3][gl][i]) / hw;
  if (d.ext) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (c8 + i < d.Co) static_cast<float*>(a.ext_out[p])[(int64_t)n * d.Co + c8 + i] = sum[i];
  } else if (d.out_f32) {
    store8(reinterpret_cast<float*>(a.abase + d.y_off) + (int64_t)n * d.Cop + c8, sum);
  } else {
    store8(reinterpret_cast<TA*>(a.abase + d.y_off) + (int64_t)n * d.Cop + c8, sum);
  }
}

// ---------------------------------------------------------------------------------
// fully connected layer: y = x W^T is a weight stream, so the reduction is split across waves
// to put the whole chip on the weight matrix.  One wave owns 32 output features x one slice of
// K x up to 32 images: per 16 reduction elements it loads its 32x16 weight block -- one
// contiguous kilobyte, the packed layout stores the blocks in the order the lanes consume them,
// so every cache line is requested exactly once -- and the 16x32 slice of x (batch in the MFMA
// column dimension, columns past the batch are zero), issues one 32x32x16 MFMA (two for fp32
// activations: hi/lo split), and finally writes its fp32 partial [batch][feature] block to the
// workspace.  Batches above 32 take one such pass per 32 images (the matrix is then streamed
// once per pass).  reduce_kernel sums the partials in a fixed order (deterministic), adds the
// bias and the residual, applies the activation and stores.
// ---------------------------------------------------------------------------------
// One wave's share of a fully connected problem: the 32 x 32 block (features of `tile` x images of `chunk`)
// reduced over slice `split` of the weight rows.  Lane l ends up with image chunk*32 + (l & 31), features
// tile*32 + 8*g + 4*(l >> 5) + t in acc[4*g + t].
template <bool WIDE>
__device__ __forceinline__ f32x16 fc_partial(const KArgs& a, const Desc& d, int batch, int tile, int split, int chunk, int lane) {
  const int steps = d.Kp / 16;
  const int per = (steps + d.splits - 1) / d.splits;
  const int s0 = split * per, s1 = min(steps, s0 + per);
  const int kq = (lane >> 5) * 8;
  // block (tile, step) of the packed matrix is 64 x 16 bytes in lane order
  const uint4* wp = reinterpret_cast<const uint4*>(a.wbase + d.w_off) + (int64_t)tile * steps * 64 + lane;
  const int n = chunk * 32 + (lane & 31);
  const bool nok = n < batch;
  const int K = d.Cp;  // flattened input length (elements), a multiple of 8
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
  constexpr int U = 8;
  for (int sb = s0; sb < s1; sb += U) {
    uint4 wv[U];
    uint4 xv[U][WIDE ? 2 : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int st = sb + u;
      const bool ok = st < s1;
      wv[u] = ok ? wp[(int64_t)st * 64] : make_uint4(0, 0, 0, 0);
      const int k = st * 16 + kq;
      const bool xok = ok && nok && k < K;
      if constexpr (WIDE) {
        const float* xp = reinterpret_cast<const float*>(a.abase + d.x_off) + (int64_t)n * K + k;
        xv[u][0] = xok ? *reinterpret_cast<const uint4*>(xp) : make_uint4(0, 0, 0, 0);
        xv[u][1] = xok ? *reinterpret_cast<const uint4*>(xp + 4) : make_uint4(0, 0, 0, 0);
      } else {
        const bf16_t* xp = reinterpret_cast<const bf16_t*>(a.abase + d.x_off) + (int64_t)n * K + k;
        xv[u][0] = xok ? *reinterpret_cast<const uint4*>(xp) : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bf16x8 wf = __builtin_bit_cast(bf16x8, wv[u]);
      if constexpr (WIDE) {
        uint4 hi, lo;
        const uint32_t* s0p = reinterpret_cast<const uint32_t*>(&xv[u][0]);
        uint32_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x0 = __uint_as_float(s0p[2 * e]), x1 = __uint_as_float(s0p[2 * e + 1]);
          const uint32_t h0 = f2bf(x0), h1 = f2bf(x1);
          h[e] = h0 | (h1 << 16);
          l[e] = pack_bf16x2(x0 - __uint_as_float(h0 << 16), x1 - __uint_as_float(h1 << 16));
        }
        hi = make_uint4(h[0], h[1], h[2], h[3]);
        lo = make_uint4(l[0], l[1], l[2], l[3]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, __builtin_bit_cast(bf16x8, lo), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, __builtin_bit_cast(bf16x8, hi), acc, 0, 0, 0);
      } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, __builtin_bit_cast(bf16x8, xv[u][0]), acc, 0, 0, 0);
      }
    }
  }
  return acc;
}

template <bool WIDE>
__global__ void __launch_bounds__(256) fc_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_FC, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int lane = threadIdx.x & 63;
  int unit = bid * 4 + (threadIdx.x >> 6);
  const int per_chunk = d.tiles_n * d.splits;
  if (unit >= per_chunk * ((batch + 31) / 32)) return;
  const int chunk = unit / per_chunk;   // which 32 images
  unit -= chunk * per_chunk;
  const int tile = unit % d.tiles_n, split = unit / d.tiles_n;
  const f32x16 acc = fc_partial<WIDE>(a, d, batch, tile, split, chunk, lane);
  const int n = chunk * 32 + (lane & 31);
  const bool nok = n < batch;
  // lane holds batch column n, features 8*g + 4*(lane/32) + t
  if (nok && d.splits == 1) {   // the whole reduction was this wave's: no partials, no reduce launch
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int fo = tile * 32 + 8 * g + 4 * (lane >> 5);
      if (fo < d.Cop)
        finish_row4<typename std::conditional<WIDE, float, bf16_t>::type>(a, d, p, n, fo, make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]));
    }
    return;
  }
  if (nok) {
    float* ws = reinterpret_cast<float*>(a.wsbase + d.ws_off) + ((int64_t)split * batch + n) * d.Cop + tile * 32;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int fo = 8 * g + 4 * (lane >> 5);
      if (tile * 32 + fo < d.Cop)
        *reinterpret_cast<float4*>(ws + fo) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
    }
  }
}

// The same problem with every slice of a tile inside one workgroup (16 waves, one slice each): the partial blocks
// meet in LDS, are summed in slice order and finished here, so a split layer whose weight matrix is small (a
// squeeze-excite gate, a classifier head: latency-bound, a handful of tiles) needs neither the partials' round
// trip through HBM nor the reduce launch.  Slices and summation order are those of fc_kernel + reduce_kernel.
template <bool WIDE>
__global__ void __launch_bounds__(1024) fc_block_kernel(KArgs a) {
  __shared__ float part[16][32][32];   // [slice][image][feature]
  int p, bid;
  if (!find_problem(a, K_FC, 1, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = bid / d.tiles_n, tile = bid % d.tiles_n;
  if (wave < d.splits) {
    const f32x16 acc = fc_partial<WIDE>(a, d, batch, tile, wave, chunk, lane);
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<float4*>(&part[wave][lane & 31][8 * g + 4 * (lane >> 5)]) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
  }
  __syncthreads();
  if (threadIdx.x >= 256) return;
  const int nl = threadIdx.x >> 3, o4 = (threadIdx.x & 7) * 4;
  const int n = chunk * 32 + nl, fo = tile * 32 + o4;
  if (n >= batch || fo >= d.Cop) return;
  float4 sum = make_float4(0, 0, 0, 0);
  for (int s = 0; s < d.splits; ++s) {   // slice order, as the reduce kernel adds them
    const float4 v = *reinterpret_cast<const float4*>(&part[s][nl][o4]);
    sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
  }
  finish_row4<typename std::conditional<WIDE, float, bf16_t>::type>(a, d, p, n, fo, sum);
}

// Finishes a split-K node (small-batch FC or a split convolution): sums the fp32 partials
// [splits][rows][Cop] in split order, adds bias (and residual), applies the activation, stores.
template <typename TA>
__global__ void __launch_bounds__(256) reduce_kernel(KArgs a) {
  int p, bid;
  if (!find_problem(a, K_REDUCE, 0, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];   // images of this problem's member in this pass
  const int q4 = d.Cop / 4;
  const int rows = batch * d.Ho * d.Wo;
  const int idx = bid * 256 + threadIdx.x;
  if (idx >= rows * q4) return;
  const int o = (idx % q4) * 4, n = idx / q4;
  const float* ws = reinterpret_cast<const float*>(a.wsbase + d.ws_off) + (int64_t)n * d.Cop + o;
  float4 sum = make_float4(0, 0, 0, 0);
  const int64_t stride = (int64_t)rows * d.Cop;
  int s = 0;
  for (; s + 8 <= d.splits; s += 8) {   // eight partials in flight, added in split order
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(ws + (s + u) * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
  }
  for (; s < d.splits; ++s) {
    const float4 v = *reinterpret_cast<const float4*>(ws + s * stride);
    sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
  }
  finish_row4<TA>(a, d, p, n, o, sum);
}

// ---------------------------------------------------------------------------------
// row copies for the request aggregator: row r of the launch goes from src[r] to dst[r]
// (the pointers travel as kernel arguments), 16 bytes per thread and step
// ---------------------------------------------------------------------------------
struct CopyArgs {
  const uint4* src[kCopyRows];
  uint4* dst[kCopyRows];
  uint32_t vecs;            // 16-byte vectors per row
  uint32_t blocks_per_row;
};

__global__ void __launch_bounds__(256) copy_rows_kernel(CopyArgs c) {
  const uint32_t row = blockIdx.x / c.blocks_per_row, part = blockIdx.x % c.blocks_per_row;
  const uint4* __restrict__ s = c.src[row];
  uint4* __restrict__ d = c.dst[row];
  for (uint32_t i = part * 256 + threadIdx.x; i < c.vecs; i += c.blocks_per_row * 256) d[i] = s[i];
}

int launch_copy_rows(const void* const* src, void* const* dst, int32_t n, uint64_t bytes, void* stream) {
  if (bytes % 16 || bytes / 16 > 0xFFFFFFFFull) return (int)hipErrorInvalidValue;
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int32_t first = 0; first < n; first += kCopyRows) {
    CopyArgs c{};
    const int32_t rows = n - first < kCopyRows ? n - first : kCopyRows;
    for (int32_t r = 0; r < rows; ++r) {
      if ((reinterpret_cast<uintptr_t>(src[first + r]) | reinterpret_cast<uintptr_t>(dst[first + r])) & 15) return (int)hipErrorInvalidValue;
      c.src[r] = static_cast<const uint4*>(src[first + r]);
      c.dst[r] = static_cast<uint4*>(dst[first + r]);
    }
    c.vecs = (uint32_t)(bytes / 16);
    c.blocks_per_row = (c.vecs + 2047) / 2048;          // a thread moves up to eight vectors
    if (c.blocks_per_row > 64) c.blocks_per_row = 64;
    if (c.blocks_per_row == 0) continue;
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)rows * c.blocks_per_row), dim3(256), 0, st, c);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return (int)hipSuccess;
}

// ---------------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------------
template <typename F>
static int go(F kernel, int blocks, int threads, const KArgs& a, hipStream_t s) {
  if (blocks <= 0) return (int)hipSuccess;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3((unsigned)threads), 0, s, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Split-K workspace of the entry point that allocates nothing (fi_run_static): one array per GPU, held from the
// moment the library's code object is loaded on that GPU until the process ends.  In host code the array's name
// is only a stand-in: its device address comes from hipGetSymbolAddress, once per device, and that address is
// what the kernels receive as KArgs::wsbase (exactly as they receive the workspace of a loaded handle).
// ---------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[FI_STATIC_SCRATCH_BYTES];

int static_scratch(void** ptr, uint64_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* per_device[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (!per_device[dev]) {   // every GPU holds its own copy of the array at its own address
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  *bytes = FI_STATIC_SCRATCH_BYTES;
  return (int)hipSuccess;
}

int launch_kernel(const Launch& L, const KArgs& args, void* stream, const std::vector<Desc>& hd) {
  if (L.kind == K_CHAIN) return launch_chain(L, args, stream, hd);
  if (L.kind == K_STEM) return launch_stem(L, args, stream, hd);
  hipStream_t s = static_cast<hipStream_t>(stream);
  KArgs a = args;
  for (int i = 0; i < L.n; ++i) a.d[i] = hd[(size_t)(L.first_desc + i)];
  int64_t blocks = 0;
  for (int i = 0; i < FI_MAX_GROUP + 1; ++i) {
    a.first_block[i] = (int32_t)blocks;
    if (i < L.n) blocks += problem_blocks(L.kind, L.tile, hd[(size_t)(L.first_desc + i)], a.batch[i]);
    if (blocks > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
  }
  const bool wb = L.wdtype == FI_BF16, ab = L.adtype == FI_BF16;
  const int nb = (int)blocks;
  // Tensors stored inside a concatenation have a pixel stride of their own: only the kernels that take one may see them.
  for (int i = 0; i < L.n; ++i) {
    const Desc& t = hd[(size_t)(L.first_desc + i)];
    if (L.kind == K_STAGE || (t.xs == t.Cp && t.ys == t.Cop)) continue;
    const bool reads = (L.kind == K_DWCONV && wb && ab && hd[(size_t)L.first_desc].vec) ||
                       ((L.kind == K_CONV_MFMA || L.kind == K_REDUCE) && (ab ? t.pre_kind != 0 : t.pre_kind == 2));   // (the reduce launch shares the node's descriptor and reads no input)
    const bool writes = ab && !t.ext && !t.out_f32 &&
                        (L.kind == K_CONV_MFMA || L.kind == K_REDUCE || (L.kind == K_DWCONV && wb && hd[(size_t)L.first_desc].vec) ||
                         ((L.kind == K_MAXPOOL || L.kind == K_AVGPOOL || L.kind == K_GATHER) && t.vec));
    if ((t.xs != t.Cp && !reads) || (t.ys != t.Cop && !writes)) return (int)hipErrorInvalidValue;
  }
  switch (L.kind) {
    case K_STAGE:
      if (wb && ab) return go(stage_kernel<bf16_t, bf16_t>, nb, 256, a, s);
      if (wb) return go(stage_kernel<bf16_t, float>, nb, 256, a, s);
      return go(stage_kernel<float, float>, nb, 256, a, s);
    case K_CONV_DIRECT:
      if (wb && ab) return go(conv_direct_kernel<bf16_t, bf16_t>, nb, 256, a, s);
      if (wb) return go(conv_direct_kernel<bf16_t, float>, nb, 256, a, s);
      return go(conv_direct_kernel<float, float>, nb, 256, a, s);
    case K_CONV_MFMA:
      if (!wb) return (int)hipErrorInvalidValue;
      if (hd[(size_t)L.first_desc].Cp == 4) {  // 4-channel model input
        if (!ab) {
          if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, true, true>, nb, 256, a, s);
          if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, true, true>, nb, 256, a, s);
          return (int)hipErrorInvalidValue;
        }
        if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, false, true>, nb, 256, a, s);
        if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, false, true>, nb, 256, a, s);
        return (int)hipErrorInvalidValue;
      }
      if (!ab && hd[(size_t)L.first_desc].pre_kind != 0) {  // fp32 activations with the squeeze-excite gate applied on the input side
        for (int i = 0; i < L.n; ++i) {
          const Desc& t = hd[(size_t)(L.first_desc + i)];
          if (t.pre_kind != 2 || t.pw_off == kNone || t.k != 1 || t.kw != 1 || t.stride != 1 || t.pad != 0 || t.pad_w != 0 || t.gin > 0 ||
              t.xs < t.Cp || t.Cp % 8 || (uint64_t)t.H * t.W * (uint64_t)t.xs * 4 * (uint64_t)a.batch[i] >= (1ull << 31))
            return (int)hipErrorInvalidValue;
        }
        if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, true, false, false, 2>, nb, 256, a, s);
        if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, true, false, false, 2>, nb, 256, a, s);
        if (L.tile == T_64x64) return go(conv_mfma_kernel<T_64x64, 64, 64, 2, 2, true, false, false, 2>, nb, 256, a, s);
        return (int)hipErrorInvalidValue;
      }
      if (!ab) {  // fp32 activations: split-bf16 inputs
        if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, true>, nb, 256, a, s);
        if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, true>, nb, 256, a, s);
        if (L.tile == T_64x64) return go(conv_mfma_kernel<T_64x64, 64, 64, 2, 2, true>, nb, 256, a, s);
        return (int)hipErrorInvalidValue;
      }
      if (hd[(size_t)L.first_desc].gin > 0) {  // grouped convolutions whose tiles walk their own groups only
        for (int i = 0; i < L.n; ++i) {
          const Desc& g = hd[(size_t)(L.first_desc + i)];
          if (g.gin <= 0 || g.gout <= 0 || g.Cp % 64 || g.splits != 1) return (int)hipErrorInvalidValue;
        }
        if (L.tile == T_256x64) return go(conv_mfma_kernel<T_256x64, 256, 64, 4, 1, false, false, true>, nb, 256, a, s);
        if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, false, false, true>, nb, 256, a, s);
        if (L.tile == T_64x64) return go(conv_mfma_kernel<T_64x64, 64, 64, 2, 2, false, false, true>, nb, 256, a, s);
        return (int)hipErrorInvalidValue;
      }
      if (hd[(size_t)L.first_desc].pre_kind != 0) {  // pointwise convolutions with a stage on their input side (per-channel affine, or gate)
        const int pk = hd[(size_t)L.first_desc].pre_kind;
        for (int i = 0; i < L.n; ++i) {
          const Desc& t = hd[(size_t)(L.first_desc + i)];
          if (t.pre_kind != pk || (pk != 1 && pk != 2) || t.pw_off == kNone || (pk == 1 && t.pb_off == kNone) ||
              t.k != 1 || t.kw != 1 || t.stride != 1 || t.pad != 0 || t.pad_w != 0 || t.gin > 0 || t.xs < t.Cp || t.Cp % 8 ||
              (uint64_t)t.H * t.W * (uint64_t)t.xs * 2 * (uint64_t)a.batch[i] >= (1ull << 31))
            return (int)hipErrorInvalidValue;
        }
#define FI_PRE_TILES(PK)                                                                                                             \
        if (L.tile == T_256x128) return go(conv_mfma_kernel<T_256x128, 256, 128, 2, 2, false, false, false, PK>, nb, 256, a, s);     \
        if (L.tile == T_256x64) return go(conv_mfma_kernel<T_256x64, 256, 64, 4, 1, false, false, false, PK>, nb, 256, a, s);        \
        if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, false, false, false, PK>, nb, 256, a, s);     \
        if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, false, false, false, PK>, nb, 256, a, s);        \
        return go(conv_mfma_kernel<T_64x64, 64, 64, 2, 2, false, false, false, PK>, nb, 256, a, s);
        if (pk == 1) { FI_PRE_TILES(1) }
        FI_PRE_TILES(2)
#undef FI_PRE_TILES
      }
      if (L.tile == T_256x128) return go(conv_mfma_kernel<T_256x128, 256, 128, 2, 2, false>, nb, 256, a, s);
      if (L.tile == T_256x64) return go(conv_mfma_kernel<T_256x64, 256, 64, 4, 1, false>, nb, 256, a, s);
      if (L.tile == T_128x128) return go(conv_mfma_kernel<T_128x128, 128, 128, 2, 2, false>, nb, 256, a, s);
      if (L.tile == T_128x128_DEEP) return go(conv_mfma_kernel<T_128x128_DEEP, 128, 128, 2, 2, false, false, false, 0, 3>, nb, 256, a, s);
      if (L.tile == T_128x64) return go(conv_mfma_kernel<T_128x64, 128, 64, 2, 2, false>, nb, 256, a, s);
      if (L.tile != T_64x64) return (int)hipErrorInvalidValue;
      return go(conv_mfma_kernel<T_64x64, 64, 64, 2, 2, false>, nb, 256, a, s);
    case K_DWCONV: {
      const bool vec = hd[(size_t)L.first_desc].vec != 0;
      if (vec && hd[(size_t)L.first_desc].tiles_n > 1) {   // the planner found one filter size and stride for the whole launch
        const int ks = hd[(size_t)L.first_desc].k, st = hd[(size_t)L.first_desc].stride;
#define FI_DW_STRIP(K, T) if (ks == K && st == T) return ab ? go(dwconv_strip_kernel<bf16_t, K, T>, nb, 256, a, s) : go(dwconv_strip_kernel<float, K, T>, nb, 256, a, s);
        FI_DW_STRIP(3, 1) FI_DW_STRIP(3, 2) FI_DW_STRIP(5, 1) FI_DW_STRIP(5, 2) FI_DW_STRIP(7, 1) FI_DW_STRIP(7, 2)
#undef FI_DW_STRIP
        return (int)hipErrorInvalidValue;
      }
      if (vec) return ab ? go(dwconv_vec_kernel<bf16_t>, nb, 256, a, s) : go(dwconv_vec_kernel<float>, nb, 256, a, s);
      if (wb && ab) return go(dwconv_kernel<bf16_t, bf16_t>, nb, 256, a, s);
      if (wb) return go(dwconv_kernel<bf16_t, float>, nb, 256, a, s);
      return go(dwconv_kernel<float, float>, nb, 256, a, s);
    }
    case K_MAXPOOL:
    case K_AVGPOOL: {
      const bool avg = L.kind == K_AVGPOOL;
      if (hd[(size_t)L.first_desc].tiles_n > 1) {   // the planner found 3x3 stride-1 windows on bf16 vectors in the whole launch
        for (int i = 0; i < L.n; ++i) {
          const Desc& t = hd[(size_t)(L.first_desc + i)];
          if (!ab || !t.vec || t.tiles_n != 4 || t.k != 3 || t.stride != 1 || t.ext) return (int)hipErrorInvalidValue;
        }
        return avg ? go(pool_strip_kernel<true>, nb, 256, a, s) : go(pool_strip_kernel<false>, nb, 256, a, s);
      }
      if (avg) return ab ? go(pool_kernel<bf16_t, true>, nb, 256, a, s) : go(pool_kernel<float, true>, nb, 256, a, s);
      return ab ? go(pool_kernel<bf16_t, false>, nb, 256, a, s) : go(pool_kernel<float, false>, nb, 256, a, s);
    }
    case K_GAP: {
      const bool vec = hd[(size_t)L.first_desc].vec != 0;
      if (vec) return ab ? go(gap_vec_kernel<bf16_t>, nb, 256, a, s) : go(gap_vec_kernel<float>, nb, 256, a, s);
      return ab ? go(gap_kernel<bf16_t>, nb, 256, a, s) : go(gap_kernel<float>, nb, 256, a, s);
    }
    case K_FC:
      if (!wb) return (int)hipErrorInvalidValue;
      if (L.tile == 1) {
        for (int i = 0; i < L.n; ++i)
          if (hd[(size_t)(L.first_desc + i)].splits < 1 || hd[(size_t)(L.first_desc + i)].splits > 16) return (int)hipErrorInvalidValue;
        return ab ? go(fc_block_kernel<false>, nb, 1024, a, s) : go(fc_block_kernel<true>, nb, 1024, a, s);
      }
      return ab ? go(fc_kernel<false>, nb, 256, a, s) : go(fc_kernel<true>, nb, 256, a, s);
    case K_REDUCE:
      return ab ? go(reduce_kernel<bf16_t>, nb, 256, a, s) : go(reduce_kernel<float>, nb, 256, a, s);
    case K_SOFTMAX:
      return go(softmax_kernel, nb, 64, a, s);
    case K_GATHER:
      return ab ? go(gather_kernel<bf16_t>, nb, 256, a, s) : go(gather_kernel<float>, nb, 256, a, s);
    case K_MUL:
      return ab ? go(mul_kernel<bf16_t>, nb, 256, a, s) : go(mul_kernel<float>, nb, 256, a, s);
    case K_CONCAT:
      return ab ? go(concat_kernel<bf16_t>, nb, 256, a, s) : go(concat_kernel<float>, nb, 256, a, s);
  }
  return (int)hipErrorInvalidValue;
}

}  // namespace fi
