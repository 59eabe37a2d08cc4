// The first convolution of an ImageNet-style member, over the 4-channel model input, 64 output channels (Section V,
// Table III): 7x7 stride 2 (the ResNet, Wide ResNet, ResNeXt, DenseNet and GoogLeNet stems), 3x3 stride 1 (VGG) or
// 3x3 stride 2 (SqueezeNet 1.1); a stride-2 one optionally with the 3x3 stride-2 max-pool (padding 0 or 1) that alone
// reads it, in one launch.
//
// The general implicit-GEMM kernel gathers this layer's reduction vectors pixel by pixel from HBM (a 4-channel
// pixel is 8 bytes, a reduction vector two filter taps) and is bound by that address work.  Here a workgroup owns a
// two-dimensional block of output pixels, brings the input patch under it into LDS once (rows of contiguous pixels,
// for stride 2 even and odd columns in planes of their own so that the reads of neighbouring output pixels are
// contiguous), and feeds the matrix cores straight from the patch: no im2col tile exists anywhere.  The 64 x 196
// (or 64 x 36) weights stay in registers as MFMA operands for as long as the workgroup lives, and a workgroup walks several
// pixel blocks (the next block's patch is requested before the current block is multiplied).
//
// The reduction order is the general kernel's (taps row-major, 4 channels per tap, 16 elements per MFMA, ascending),
// bias, activation and the one rounding to bf16 are its operations, and the max-pool combines its taps with the pooling
// kernel's operation in the pooling kernel's order: the outputs are the same bits as the separate launches'.
#include <hip/hip_runtime.h>

#include "fi_device.h"

namespace fi {
namespace {

constexpr int CO = 64;           // output channels
constexpr int OS = 72;           // bf16 elements per pixel row of the LDS output tile (144 bytes: 16-byte reads hit all banks)

// SK: filter side, SS: stride.
template <int SK, int SS, bool POOL>
struct Geo {
  static constexpr int LAST_TAP = SK * SK - 1;
  static constexpr int KP = (SK * SK * 4 + 31) / 32 * 32;               // packed weight row: 4 channels per tap, rounded up to 32 elements
  static constexpr int KSTEPS = (SK * SK * 4 + 15) / 16;                // 16-element reduction steps that hold a real tap
  // steps whose weight fragments stay in registers; the others wait in LDS (the registers they would take are the ones
  // the tile loop is short of)
  static constexpr int KREG = KSTEPS < 12 ? KSTEPS : 12;
  // convolution outputs one block covers: with the pool, 15 x 17 of them are what 7 x 8 pooled pixels read
  static constexpr int CH = POOL ? 15 : 16, CW = POOL ? 17 : 16;
  static constexpr int NPX = CH * CW;                                   // <= 256: eight 32-pixel MFMA column blocks
  static constexpr int PH = (CH - 1) * SS + SK, PW = (CW - 1) * SS + SK;  // the input patch under them
  // Stride 2: a patch row is an even-column plane and an odd-column plane of HALF pixels each.  With the pool 8 bytes more:
  // the lanes that take the block's 17th column read one pixel per row, and rows 656 instead of 640 bytes apart spread
  // them over the banks.  Stride 1: the pixels of a row in their order.
  static constexpr int HALF = ((PW + 1) / 2 + 3) / 4 * 4;
  static constexpr int ROWB = SS == 2 ? 2 * HALF * 8 + (POOL ? 8 : 0) : (PW * 8 + 15) / 16 * 16;
  static constexpr int NPATCH = PH * PW;
  static constexpr int SLOTS = (NPATCH + 255) / 256;                    // patch pixels a thread brings in
  static constexpr int PATCH_BYTES = PH * ROWB;
  static constexpr int ZERO_AT = (PATCH_BYTES + 15) / 16 * 16;          // 16 zero bytes: taps past the filter, patch slots past the patch
  static constexpr int BIAS_AT = ZERO_AT + 16;
  static constexpr int WLDS_AT = BIAS_AT + CO * 4;                      // weight fragments of steps KREG.., [step][32-channel block][lane]
  static constexpr int OUT_AT = WLDS_AT + (KSTEPS - KREG) * 2 * 64 * 16;
  // where pixel (pr, pc) of the patch sits in LDS
  static constexpr int at(int pr, int pc) { return SS == 2 ? pr * ROWB + (pc & 1) * HALF * 8 + (pc >> 1) * 8 : pr * ROWB + pc * 8; }
  static constexpr int LDS_BYTES = OUT_AT + 256 * OS * 2;
  static constexpr int TPH = 7, TPW = 8;                                // pooled pixels per block
  static_assert(SS == 1 || SS == 2, "strides 1 and 2");
  static_assert(!POOL || SS == 2, "the pool's block geometry is the stride-2 one");
  static_assert((PW + 1) / 2 <= HALF, "a patch row fits its two planes");
  static_assert(NPX <= 256, "eight 32-pixel blocks");
  static_assert(OUT_AT % 16 == 0 && WLDS_AT % 16 == 0 && BIAS_AT % 16 == 0, "16-byte LDS accesses are aligned");
  static_assert(KSTEPS - KREG <= 4, "one wave parks one step's fragments");
  static_assert(PW < 255, "patch columns fit 8 bits");
};

// Byte offset of filter tap `tap` (row-major) from an output pixel's window origin in the LDS patch.
template <int SK, int SS, bool POOL>
__device__ __forceinline__ constexpr int tap_offset(int tap) { return Geo<SK, SS, POOL>::at(tap / SK, tap % SK); }

// One descriptor per problem.  Convolution fields as for any convolution (H, W, Cp = 4, k = kw = SK, stride SS, pad,
// pad_w, act, w_off, b_off, Kp = 224 or 64); gin x gout is the convolution's output (height x width); Ho x Wo is what is
// stored at y_off: the same without the pool, the pooled size with it (3x3 windows, stride 2, padding pre_act = 0 or 1,
// every window starting inside the convolution's output: floor or ceil mode); tiles_n = workgroups that share the problem.
// CLAMP6: the launch holds a ReLU6 (otherwise the upper clamp is not applied at all).
template <int SK, int SS, bool POOL, bool CLAMP6>
__global__ void __launch_bounds__(256, 2) stem_kernel(KArgs a) {
  using G = Geo<SK, SS, POOL>;
  constexpr int KSTEPS = G::KSTEPS, KREG = G::KREG, STEM_KP = G::KP, LAST_TAP = G::LAST_TAP;
  __shared__ __attribute__((aligned(16))) uint8_t smem[G::LDS_BYTES];
  int p, bid;
  if (!find_problem_at(a, (int)blockIdx.x, p, bid)) return;
  const Desc d = a.d[p];
  const int batch = a.batch[p];
  const int Hc = d.gin, Wc = d.gout;
  const int pool_pad = d.pre_act;             // (with the pool: its padding, 0 or 1)
  const int ty = POOL ? (d.Ho + G::TPH - 1) / G::TPH : (Hc + G::CH - 1) / G::CH;
  const int tx = POOL ? (d.Wo + G::TPW - 1) / G::TPW : (Wc + G::CW - 1) / G::CW;
  const int ntiles = batch * ty * tx;
  const int nwg = min(d.tiles_n, ntiles);     // workgroups of this problem (the launch counted them the same way)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool upper = lane >= 32;              // lanes 32-63 hold reduction elements 8-15 of a step

  const uint8_t* const xbase = a.abase + d.x_off;
  const int image_bytes = d.H * d.W * 8;
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(a.wbase + d.w_off), 0, CO * STEM_KP * 2, 0x00020000);
  // (the stored tensor may sit inside a concatenation's: its pixels are then ys, not 64, channels apart)
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      a.abase + d.y_off, 0, batch > 0 ? (int)((((int64_t)batch * d.Ho * d.Wo - 1) * d.ys + CO) * 2) : 0, 0x00020000);
  const bool stream_out = (int64_t)batch * d.Ho * d.Wo * CO * 2 > (int64_t)STREAM_OUT_BYTES;

  // the weights: the MFMA operand fragments of every reduction step, for both 32-channel blocks
  bf16x8 bw[KREG][2];
#pragma unroll
  for (int ks = 0; ks < KREG; ++ks)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      bw[ks][j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
          wres, (uint32_t)(((j * 32 + (lane & 31)) * STEM_KP + ks * 16 + (upper ? 8 : 0)) * 2), 0, 0));
  if (wave < KSTEPS - KREG) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      *reinterpret_cast<u32x4*>(smem + G::WLDS_AT + ((wave * 2 + j) * 64 + lane) * 16) = __builtin_amdgcn_raw_buffer_load_b128(
          wres, (uint32_t)(((j * 32 + (lane & 31)) * STEM_KP + (KREG + wave) * 16 + (upper ? 8 : 0)) * 2), 0, 0);
  }
  if (tid < CO / 4)
    *reinterpret_cast<float4*>(smem + G::BIAS_AT + tid * 16) = *reinterpret_cast<const float4*>(a.wbase + d.b_off + tid * 16);
  if (tid == 0) *reinterpret_cast<uint4*>(smem + G::ZERO_AT) = make_uint4(0, 0, 0, 0);

  // This thread's patch pixels: slot j is pixel tid + 256 j of the patch, row-major.  Per slot: the pixel's byte offset from
  // the patch origin in the image, and (one register) its column in the patch and where it goes in LDS (a slot past the
  // patch reads zeros and writes them to the zero slot).
  int slot_rel[G::SLOTS], slot_at[G::SLOTS];   // slot_at: LDS byte offset << 8 | patch column (255: a column no image has)
#pragma unroll
  for (int j = 0; j < G::SLOTS; ++j) {
    const int i = tid + 256 * j;
    const int pr = i / G::PW, pc = i - pr * G::PW;
    const bool in_patch = i < G::NPATCH;
    slot_rel[j] = (pr * d.W + pc) * 8;
    slot_at[j] = in_patch ? (G::at(pr, pc) << 8) | pc : (G::ZERO_AT << 8) | 255;
  }
  // Window origins in the LDS patch of the two 32-pixel blocks this wave multiplies.  Lanes 32-63 read the tap two
  // places after the one lanes 0-31 read; seen from a tap at column t of the filter that is a fixed distance on in the
  // same filter row (t <= SK - 3), or wraps to the next row (t = SK - 2 and t = SK - 1: two other distances).  One base per case with the lane half's
  // distance already in it leaves every read as base + a constant the instruction carries.  The fourth base sends
  // lanes 32-63 to the zero slot: the last step's upper half lies past the filter.
  // Which pixels: 16 neighbouring lanes take 16 neighbouring pixels of one row of the block (their reads are 128
  // contiguous bytes of a plane: every bank once).  Without the pool that is all 16 x 16 pixels; with it, rows of 17:
  // fifteen half-groups take columns 0-15 of the fifteen rows, the sixteenth takes column 16 of all of them.
  int win[2][4], out_at[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int hg = wave * 4 + i * 2 + ((lane & 31) >> 4), l16 = lane & 15;
    int cy = hg, cx = l16;
    bool real = true;
    if constexpr (POOL) {
      if (hg == G::CH) { cy = l16; cx = G::CW - 1; real = l16 < G::CH; }
      cy = real ? cy : 0;
    }
    out_at[i] = (real ? cy * G::CW + cx : 255) * (OS / 8); // the pixel's row in the LDS output tile, in 16-byte pieces (row 255: nobody reads it)
    const int w0 = (SS * cy) * G::ROWB + cx * 8;   // (stride 2: output column cx starts at patch column 2 cx, element cx of the even plane)
    win[i][0] = w0 + (upper ? tap_offset<SK, SS, POOL>(2) - tap_offset<SK, SS, POOL>(0) : 0);
    win[i][1] = w0 + (upper ? tap_offset<SK, SS, POOL>(SK) - tap_offset<SK, SS, POOL>(SK - 2) : 0);
    win[i][2] = w0 + (upper ? tap_offset<SK, SS, POOL>(SK + 1) - tap_offset<SK, SS, POOL>(SK - 1) : 0);
    win[i][3] = upper ? G::ZERO_AT - tap_offset<SK, SS, POOL>(LAST_TAP) : w0;
  }
  // identity / ReLU / ReLU6 as max and min against bounds that are NaN where there is none (max / min return the other
  // operand): the general kernel's two instructions, with the min left out where no problem of the launch has a ReLU6
  uint32_t lo_b = d.act == FI_ACT_NONE ? 0x7FC00000u : 0u, hi_b = d.act == FI_ACT_RELU6 ? 0x40C00000u : 0x7FC00000u;
  asm volatile("" : "+v"(lo_b), "+v"(hi_b));
  const float act_lo = __uint_as_float(lo_b), act_hi = __uint_as_float(hi_b);

  u32x2 pv[G::SLOTS];
  // With the pool, a tile's two output vectors per thread leave one iteration late, just before the next patch is
  // requested: a store issued after those loads would have to complete before the loads' data may be used (one
  // in-order counter covers both), and the wait for the patch would be a wait for the store's acknowledgement.
  u32x4 late[2] = {};
  uint32_t late_off[2] = {OOB, OOB};          // (nothing to store yet: out of range, dropped)
  int n, by, bx;   // image and block position of the tile whose patch is in flight
#define FI_TILE_POS(T)                                                                            \
  {                                                                                               \
    const int per = ty * tx;                                                                      \
    n = (T) / per;                                                                                \
    const int rem = (T) - n * per;                                                                \
    by = rem / tx;                                                                                \
    bx = rem - by * tx;                                                                           \
  }
  // first convolution output of block (by, bx)
#define FI_ORIGIN(CY0, CX0)                                                                       \
  const int CY0 = POOL ? by * G::TPH * 2 - pool_pad : by * G::CH, CX0 = POOL ? bx * G::TPW * 2 - pool_pad : bx * G::CW;
  // The patch of block (n, by, bx) through a buffer resource that covers image n alone: a row above or below the image
  // is out of its range and reads zero by itself; a column left or right of the image would land in a neighbouring row
  // and takes the out-of-range offset.  (LIVE false: an empty resource, everything reads zero.)
#define FI_FETCH_PATCH(LIVE)                                                                      \
  {                                                                                               \
    FI_ORIGIN(cy0, cx0)                                                                           \
    const int iy0 = cy0 * SS - d.pad, ix0 = cx0 * SS - d.pad_w;                                   \
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(                        \
        const_cast<uint8_t*>(xbase + (int64_t)n * image_bytes), 0, (LIVE) ? image_bytes : 0, 0x00020000); \
    const int origin = (iy0 * d.W + ix0) * 8;                                                     \
    _Pragma("unroll") for (int j = 0; j < G::SLOTS; ++j) {                                        \
      const int pc = slot_at[j] & 255;                                                            \
      const bool col_ok = pc != 255 && (uint32_t)(ix0 + pc) < (uint32_t)d.W;                      \
      pv[j] = __builtin_amdgcn_raw_buffer_load_b64(xres, col_ok ? (uint32_t)(origin + slot_rel[j]) : OOB, 0, 0); \
    }                                                                                             \
  }

  int t = bid;
  FI_TILE_POS(t)
  FI_FETCH_PATCH(t < ntiles)
  for (; t < ntiles; t += nwg) {
    const int cn = n, cby = by, cbx = bx;     // the tile being multiplied
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j) *reinterpret_cast<u32x2*>(smem + (slot_at[j] >> 8)) = pv[j];
    __syncthreads();
    if constexpr (POOL) {
#pragma unroll
      for (int j = 0; j < 2; ++j) __builtin_amdgcn_raw_buffer_store_b128(late[j], yres, late_off[j], 0, 0);
    }
    {
      const int tn = t + nwg;
      FI_TILE_POS(tn < ntiles ? tn : t)
      FI_FETCH_PATCH(tn < ntiles)             // in flight while this tile is multiplied
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    // operand fragments straight from the patch, one step ahead of the multiplies that use them (the scheduling
    // barriers keep the compiler from hoisting every step's reads to the top, which costs more registers than there are)
#define FI_READ_A(KS, AF)                                                                         \
  _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                 \
    u32x4 v;                                                                                      \
    _Pragma("unroll") for (int h = 0; h < 2; ++h) { /* elements 0-3: one tap, elements 4-7: the next */ \
      const int tap = 4 * (KS) + h;           /* what lanes 0-31 read; lanes 32-63: tap + 2 */    \
      if (tap > LAST_TAP) {                                                                       \
        v[2 * h] = v[2 * h + 1] = 0u;                                                             \
      } else {                                                                                    \
        const int col = tap % SK;                                                                 \
        const int base = tap + 2 > LAST_TAP ? 3 : col <= SK - 3 ? 0 : col == SK - 2 ? 1 : 2;      \
        const u32x2 half = *reinterpret_cast<const u32x2*>(smem + win[i][base] + tap_offset<SK, SS, POOL>(tap)); \
        v[2 * h] = half[0];                                                                       \
        v[2 * h + 1] = half[1];                                                                   \
      }                                                                                           \
    }                                                                                             \
    (AF)[i] = __builtin_bit_cast(bf16x8, v);                                                      \
  }
    bf16x8 af[2][2], wl[2];
    FI_READ_A(0, af[0])
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      if (ks + 1 < KSTEPS) { FI_READ_A(ks + 1, af[(ks + 1) & 1]) }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ks < KREG ? bw[ks < KREG ? ks : 0][j] : wl[j], af[ks & 1][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 >= KREG && ks + 1 < KSTEPS) {   // the next step's weights from LDS, into registers this step's multiplies have read
#pragma unroll
        for (int j = 0; j < 2; ++j) wl[j] = *reinterpret_cast<const bf16x8*>(smem + G::WLDS_AT + (((ks + 1 - KREG) * 2 + j) * 64 + lane) * 16);
      }
    }
#undef FI_READ_A

    // Bias, activation, the one rounding.  A lane holds, for one pixel, runs of 4 consecutive channels; the two halves of
    // the wave exchange runs so that each ends with 8 consecutive channels, parked with one 16-byte write.
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float4 b[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) b[g] = *reinterpret_cast<const float4*>(smem + G::BIAS_AT + (j * 32 + 8 * g + (upper ? 4 : 0)) * 4);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        uint32_t pk[4][2], frag[2][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4] = {acc[i][j][4 * g] + b[g].x, acc[i][j][4 * g + 1] + b[g].y, acc[i][j][4 * g + 2] + b[g].z, acc[i][j][4 * g + 3] + b[g].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = fmaxf(v[e], act_lo);
            if constexpr (CLAMP6) v[e] = fminf(v[e], act_hi);
          }
          pk[g][0] = pack_bf16x2(v[0], v[1]);
          pk[g][1] = pack_bf16x2(v[2], v[3]);
        }
        runs_to_fragments(pk, frag);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const u32x4 q = {frag[half][0], frag[half][1], frag[half][2], frag[half][3]};
          reinterpret_cast<u32x4*>(smem + G::OUT_AT)[out_at[i] + j * 4 + 2 * half + (upper ? 1 : 0)] = q;
        }
      }
    }
    __syncthreads();

    {
      const int n = cn, by = cby, bx = cbx;
      FI_ORIGIN(cy0, cx0)
      if constexpr (!POOL) {
        // every pixel row (64 channels, 128 bytes) leaves as eight 16-byte pieces of neighbouring threads
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int v = tid + 256 * j;
          const int px = v >> 3, c8 = (v & 7) * 8;
          const int cy = cy0 + px / G::CW, cx = cx0 + px % G::CW;
          const bool ok = cy < Hc && cx < Wc;
          const u32x4 q = reinterpret_cast<const u32x4*>(smem + G::OUT_AT)[px * (OS / 8) + (v & 7)];
          const uint32_t off = ok ? (uint32_t)((((n * Hc + cy) * Wc + cx) * d.ys + c8) * 2) : OOB;
          if (stream_out) __builtin_amdgcn_raw_buffer_store_b128(q, yres, off, 0, 2);
          else __builtin_amdgcn_raw_buffer_store_b128(q, yres, off, 0, 0);
        }
      } else {
        // 7 x 8 pooled pixels x eight 8-channel vectors.  The taps of a window in (row, column) order, combined with the
        // pooling kernel's operation.  A tap outside the convolution's output (the pool's padding) is not skipped but
        // moved onto the nearest row / column inside it, which lies in the same window: the maximum sees one of its
        // values twice and is the same; so is a tap that hangs over the far border in ceil mode.  (Positions relative to
        // the block: rows ly_lo..ly_hi, columns lx_lo..lx_hi exist.)
        const int ly_lo = cy0 < 0 ? -cy0 : 0, ly_hi = min(G::CH - 1, Hc - 1 - cy0);
        const int lx_lo = cx0 < 0 ? -cx0 : 0, lx_hi = min(G::CW - 1, Wc - 1 - cx0);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int v = tid + 256 * j;
          const int pp = v >> 3, c8 = (v & 7) * 8;
          const bool live = pp < G::TPH * G::TPW;
          const int ph = live ? pp >> 3 : 0, pw = pp & 7;
          int row_at[3], col_at[3];
#pragma unroll
          for (int r = 0; r < 3; ++r) {
            row_at[r] = min(max(2 * ph + r, ly_lo), ly_hi) * (G::CW * OS / 8);   // (16-byte pieces)
            col_at[r] = min(max(2 * pw + r, lx_lo), lx_hi) * (OS / 8) + (v & 7);
          }
          float best[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
          for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
              const u32x4 q = reinterpret_cast<const u32x4*>(smem + G::OUT_AT)[row_at[r] + col_at[s]];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                best[2 * e] = fmaxf(best[2 * e], __uint_as_float(q[e] << 16));
                best[2 * e + 1] = fmaxf(best[2 * e + 1], __uint_as_float(q[e] & 0xFFFF0000u));
              }
            }
          u32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e)   // the maxima are bf16 values already: packing is exact
            o[e] = (__float_as_uint(best[2 * e]) >> 16) | (__float_as_uint(best[2 * e + 1]) & 0xFFFF0000u);
          const int oy = by * G::TPH + ph, ox = bx * G::TPW + pw;
          const bool st_ok = live && oy < d.Ho && ox < d.Wo;
          late[j] = o;
          late_off[j] = st_ok ? (uint32_t)((((n * d.Ho + oy) * d.Wo + ox) * d.ys + c8) * 2) : OOB;
        }
      }
    }
    __syncthreads();   // the output tile and the patch are free again
  }
  if constexpr (POOL) {
#pragma unroll
    for (int j = 0; j < 2; ++j) __builtin_amdgcn_raw_buffer_store_b128(late[j], yres, late_off[j], 0, 0);
  }
#undef FI_TILE_POS
#undef FI_ORIGIN
#undef FI_FETCH_PATCH
}

}  // namespace

// Workgroups of one problem of a stem launch: every block of output pixels at most once, Desc.tiles_n at most.
int stem_blocks(int tile, const Desc& d, int batch) {
  const bool pool = (tile & 1) != 0;
  const int ty = pool ? (d.Ho + 6) / 7 : (d.gin + 15) / 16;
  const int tx = pool ? (d.Wo + 7) / 8 : (d.gout + 15) / 16;
  const int64_t tiles = (int64_t)batch * ty * tx;
  return (int)std::min<int64_t>(tiles, d.tiles_n);
}

int launch_stem(const Launch& L, const KArgs& args, void* stream, const std::vector<Desc>& hd) {
  const bool pool = (L.tile & 1) != 0;
  const int geom = L.tile >> 1;
  if (L.wdtype != FI_BF16 || L.adtype != FI_BF16 || L.tile < 0 || geom > 2 || (pool && geom == 1) || L.n < 1 || L.n > FI_MAX_GROUP) return (int)hipErrorInvalidValue;
  const int sk = geom == 0 ? 7 : 3, ss = geom == 1 ? 1 : 2;
  const int kp = (sk * sk * 4 + 31) / 32 * 32;
  KArgs a = args;
  int64_t blocks = 0;
  for (int i = 0; i < FI_MAX_GROUP + 1; ++i) {
    a.first_block[i] = (int32_t)blocks;
    if (i >= L.n) continue;
    const Desc& t = hd[(size_t)(L.first_desc + i)];
    a.d[i] = t;
    // what the kernel takes for granted
    if (t.k != sk || t.kw != sk || t.stride != ss || t.Cp != 4 || t.Kp != kp || t.Co != CO || t.Cop != CO || t.ys < CO || t.ys % 8 || t.xs != 4 ||
        t.act < 0 || t.act > FI_ACT_RELU6 || t.ext || t.out_f32 || t.splits != 1 || t.r_off != kNone || t.tiles_n < 1 ||
        t.pad < 0 || t.pad > sk / 2 || t.pad_w < 0 || t.pad_w > sk / 2 || t.x_off == kNone || t.y_off == kNone || t.w_off == kNone || t.b_off == kNone)
      return (int)hipErrorInvalidValue;
    if (t.H + 2 * t.pad < sk || t.W + 2 * t.pad_w < sk) return (int)hipErrorInvalidValue;
    if (t.gin != (t.H + 2 * t.pad - sk) / ss + 1 || t.gout != (t.W + 2 * t.pad_w - sk) / ss + 1 || t.gin < 1 || t.gout < 1) return (int)hipErrorInvalidValue;
    if (pool) {   // every pooling window starts inside the convolution's output
      if (t.pre_act < 0 || t.pre_act > 1 || t.Ho < 1 || t.Wo < 1 || (t.Ho - 1) * 2 - t.pre_act >= t.gin || (t.Wo - 1) * 2 - t.pre_act >= t.gout)
        return (int)hipErrorInvalidValue;
    } else if (t.Ho != t.gin || t.Wo != t.gout) return (int)hipErrorInvalidValue;
    // 32-bit byte offsets through buffer resources
    if ((uint64_t)a.batch[i] * t.H * t.W * 8 >= (1ull << 31) || (uint64_t)a.batch[i] * t.Ho * t.Wo * t.ys * 2 >= (1ull << 31)) return (int)hipErrorInvalidValue;
    blocks += stem_blocks(L.tile, t, a.batch[i]);
    if (blocks > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
  }
  if (blocks == 0) return (int)hipSuccess;
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool clamp6 = false;
  for (int i = 0; i < L.n; ++i) clamp6 = clamp6 || hd[(size_t)(L.first_desc + i)].act == FI_ACT_RELU6;
  const dim3 grid((unsigned)blocks), wg(256);
#define FI_STEM_GO(SK_, SS_, POOL_)                                                               \
  {                                                                                               \
    if (clamp6) hipLaunchKernelGGL((stem_kernel<SK_, SS_, POOL_, true>), grid, wg, 0, s, a);      \
    else hipLaunchKernelGGL((stem_kernel<SK_, SS_, POOL_, false>), grid, wg, 0, s, a);            \
  }
  if (geom == 0 && pool) FI_STEM_GO(7, 2, true)
  else if (geom == 0) FI_STEM_GO(7, 2, false)
  else if (geom == 1) FI_STEM_GO(3, 1, false)
  else if (pool) FI_STEM_GO(3, 2, true)
  else FI_STEM_GO(3, 2, false)
#undef FI_STEM_GO
  return (int)hipGetLastError();
}

}  // namespace fi
