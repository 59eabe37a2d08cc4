// Chained convolutions of one member in ONE launch (gfx950, wave64, MFMA).
//
// Algorithm 1's inference loop evaluates phi(sum u x) node by node; nothing in it says that a node's output has to
// travel through device memory before the next node reads it.  A bottleneck block is   k x k conv (A) -> 1x1 conv
// (B, + residual) -> [next block's] 1x1 conv (C),   and B and C are pointwise: output pixel m of B and of C depends
// on pixel m of A's output only.  A workgroup that owns 128 output pixels of A can therefore finish those pixels
// of B and C as well: A's output never leaves the registers, B's output is written once (the next block needs it
// as its residual) and is not read back for C.  Per block that is 10 of the 16 activation passes over memory that
// three separate launches make, and one launch instead of three.
//
// Every product-sum is accumulated exactly as conv_mfma_kernel accumulates it (same MFMA instruction, same operand
// slots, reduction tiles in ascending order from a zero accumulator; bias, residual, activation and the single
// rounding to bf16 in the same order), so a chained node's output has the bits of the node launched alone.
//
// Layout of the work: 4 waves, each owns 32 of the tile's 128 pixel rows through all three GEMMs (so that a row's
// values never have to cross waves).  With the weights as the first MFMA operand a lane ends a GEMM holding, for
// pixel (lane & 31), runs of 4 consecutive channels at 8g + 4(lane >> 5); the next GEMM wants, for the same pixel,
// 8 consecutive reduction elements at 16s + 8(lane >> 5).  The two halves of the wave exchange the runs they lack
// with v_permlane32_swap: the intermediate tile goes from accumulators to operand registers without touching LDS.
// Weights (shared by the 4 waves) are staged through LDS as in conv_mfma_kernel; residual rows and output rows
// pass through a per-wave LDS patch so that they cross HBM as 16-byte pieces of contiguous rows.
#include <hip/hip_runtime.h>

#include <vector>

#include "fi_device.h"
#include "fi_internal.h"

namespace fi {

typedef u32x4 __attribute__((may_alias)) u32x4_a;
typedef u32x2 __attribute__((may_alias)) u32x2_a;

__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

// W1: output channels of A = reduction length of B (64 or 128).  N3: output channels of C (64 or 128), 0 = no C.
// SMOOTH: some node of the launch has an activation beyond identity / ReLU / ReLU6 (the variant without them keeps
// its epilogues free of branches).
// The launch's problems are triples of descriptors: a.d[3p] = A, a.d[3p + 1] = B, a.d[3p + 2] = C.
template <int W1, int N3, bool SMOOTH>
__global__ void __launch_bounds__(256, 2) chain_mfma_kernel(KArgs a) {
  constexpr int BM = 128;
  constexpr int NI1 = W1 / 32, NI3 = N3 > 0 ? N3 / 32 : 1;
  constexpr int KT2 = W1 / 64;                 // reduction tiles of B
  constexpr int PS = 128 + 8;                  // patch row stride (bf16 elements): 272-byte rows, 16-byte aligned
  constexpr int STAGE_A = BM * LDS_STRIDE * 2; // bytes
  constexpr int PATCHES = 4 * 32 * PS * 2;
  constexpr int REGION0 = STAGE_A > PATCHES ? STAGE_A : PATCHES;   // A tiles during the first GEMM, the waves' patches afterwards
  constexpr int STAGE_B = 128 * LDS_STRIDE * 2;
  constexpr int MAXN2 = 1024;                  // widest B the bias table holds (the host checks)
  constexpr int BIAS = (W1 + MAXN2 + (N3 > 0 ? N3 : 0)) * 4;   // the three bias vectors, read by every lane in every epilogue
  constexpr bool EARLY = W1 == 64 && N3 == 64;  // registers to spare: every weight tile a chunk needs is requested before the epilogue before it
  __shared__ __attribute__((aligned(16))) uint8_t smem[REGION0 + STAGE_B + BIAS];
  bf16_t* const As = reinterpret_cast<bf16_t*>(smem);
  bf16_t* const Bs = reinterpret_cast<bf16_t*>(smem + REGION0);
  float* const bias1 = reinterpret_cast<float*>(smem + REGION0 + STAGE_B);
  float* const bias2 = bias1 + W1;
  float* const bias3 = bias2 + MAXN2;

  int p, bid;
  if (!find_problem_at(a, xcd_contiguous((int)blockIdx.x, (int)gridDim.x), p, bid)) return;
  const Desc& d1 = a.d[3 * p];
  const Desc& d2 = a.d[3 * p + 1];
  const Desc& d3 = a.d[3 * p + 2];
  const int batch = a.batch[p];
  const int M = batch * d1.Ho * d1.Wo;
  const int m0 = bid * BM;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lp = lane & 31, lh = lane >> 5;   // pixel row inside the wave's block, half of the wave

  // ---- first GEMM: implicit-GEMM convolution, staged as in conv_mfma_kernel -----------------------------
  const int Cp = d1.Cp, Wd = d1.W, kw = d1.kw;
  const bf16_t* __restrict__ w1 = reinterpret_cast<const bf16_t*>(a.wbase + d1.w_off);
  const int x_bytes = (int)((int64_t)batch * d1.H * d1.W * Cp * 2);
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.abase + d1.x_off), 0, batch > 0 ? x_bytes : 0, 0x00020000);
  const int srow = tid >> 3, kvec = (tid & 7) * 8;
  int a_row[4], a_rc[4];
  {
    const float inv_wo = 1.0f / (float)d1.Wo, inv_ho = 1.0f / (float)d1.Ho;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + srow + 32 * i;
      const bool ok = m < M;
      const int mm = ok ? m : 0;
      const int t = fast_div(mm, d1.Wo, inv_wo);
      const int q = mm - t * d1.Wo;
      const int n = fast_div(t, d1.Ho, inv_ho);
      const int pp = t - n * d1.Ho;
      const int ih0 = pp * d1.stride - d1.pad, iw0 = q * d1.stride - d1.pad_w;
      a_row[i] = ((n * d1.H + ih0) * Wd + iw0) * Cp * 2;
      const int rc = (int)(taps_inside(ih0, d1.k, d1.H) | (taps_inside(iw0, kw, Wd) << 16));
      a_rc[i] = ok ? rc : 0;   // rows past M read as zero
    }
  }
  const u32x4* b1_ptr[NI1];
#pragma unroll
  for (int i = 0; i < NI1; ++i) b1_ptr[i] = reinterpret_cast<const u32x4*>(w1 + (int64_t)(srow + 32 * i) * d1.Kp + kvec);
  const bf16_t* __restrict__ w2 = reinterpret_cast<const bf16_t*>(a.wbase + d2.w_off);
  const bf16_t* __restrict__ w3 = N3 > 0 ? reinterpret_cast<const bf16_t*>(a.wbase + d3.w_off) : nullptr;
  const int Kp3 = N3 > 0 ? d3.Kp : 0;
  const int nchunks = d2.Co / 128;

  u32x4 bv[4];
  // a [rows x 64] tile of a weight matrix with row length kp: rows row0 + (srow + 32 i), reduction elements k0 + kvec ..
#define FI_FETCH_B(W, KP, ROW0, K0, NV)                                                                      \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < (NV); ++i)                                                         \
        bv[i] = *reinterpret_cast<const u32x4*>((W) + (int64_t)((ROW0) + srow + 32 * i) * (KP) + (K0) + kvec); \
  }
#define FI_PARK_B(NV)                                                                                        \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < (NV); ++i)                                                         \
        *reinterpret_cast<u32x4*>(&Bs[(srow + 32 * i) * LDS_STRIDE + kvec]) = bv[i];                         \
  }
  // What the later phases wait for first is requested before anything else: the first tile of B's weights and the
  // residual rows of B's first chunk (32 rows x 256 bytes per wave, 16 bytes per lane and pass).
  // Residual rows in and output rows out go through buffer resources that end with the tensor's last row: a row past
  // M reads as zero and is not written, without a branch (the epilogues stay in one basic block each, so that their
  // LDS reads, loads and stores are issued in batches instead of one wait apiece).
  const bool has_res = d2.r_off != kNone;
  const int mw = m0 + wave * 32;                                         // first row of this wave
  const int cop2 = d2.Cop, ys2 = d2.ys;
  const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(a.abase + (has_res ? d2.r_off : 0)), 0, has_res && M > 0 ? (int)((int64_t)M * cop2 * 2) : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t y2res = __builtin_amdgcn_make_buffer_rsrc(
      a.abase + d2.y_off, 0, M > 0 ? (int)((((int64_t)M - 1) * ys2 + cop2) * 2) : 0, 0x00020000);
  // this lane's 16-byte piece of a 128-channel row block: rows (lane >> 4) + 4 it, channels 8 (lane & 15) ..
  const int prow = lane >> 4, pcol = (lane & 15) * 8;
  const uint32_t r_off0 = (uint32_t)(((mw + prow) * cop2 + pcol) * 2), r_step = (uint32_t)(4 * cop2 * 2);
  const uint32_t y_off0 = (uint32_t)(((mw + prow) * ys2 + pcol) * 2), y_step = (uint32_t)(4 * ys2 * 2);
  u32x4 rv[8];
#define FI_FETCH_RES_PART(CH, IT0, IT1)                                                                      \
  {                                                                                                          \
    _Pragma("unroll") for (int it = (IT0); it < (IT1); ++it)                                                 \
        rv[it] = __builtin_amdgcn_raw_buffer_load_b128(rres, r_off0 + it * r_step + (CH) * 256, 0, 0);       \
  }
#define FI_FETCH_RES(CH) FI_FETCH_RES_PART(CH, 0, 8)
  // The chains whose third convolution has 128 channels have no registers for a whole residual block next to B's
  // accumulators: RV_EARLY of its eight vectors travel ahead (during B's multiplies, or from the chunk before), the rest
  // is requested when the multiplies are done.  (A request for all eight the register allocator answers with spills,
  // and a spilled load is waited for on the spot, one after the other.)
  constexpr int RV_EARLY = N3 == 128 ? (W1 == 128 ? 4 : 7) : 8;
  FI_FETCH_B(w2, W1, 0, 0, 4)
  // The bias vectors travel to LDS through registers: every load is requested here, in one batch, and parked after the
  // first GEMM (one round trip hidden behind it instead of three in a row in front of it).
  constexpr int NB2 = MAXN2 / 256;
  float bq1, bq2[NB2], bq3 = 0.0f;
  {
    const float* g1 = reinterpret_cast<const float*>(a.wbase + d1.b_off);
    const float* g2 = reinterpret_cast<const float*>(a.wbase + d2.b_off);
    const int n2 = d2.Co;
    bq1 = g1[tid < W1 ? tid : 0];
#pragma unroll
    for (int i = 0; i < NB2; ++i) bq2[i] = g2[tid + 256 * i < n2 ? tid + 256 * i : 0];
    if constexpr (N3 > 0) bq3 = reinterpret_cast<const float*>(a.wbase + d3.b_off)[tid < N3 ? tid : 0];
  }
  constexpr bool AHEAD = W1 == 64 || N3 == 0;   // the next chunk's residual is requested while this chunk is finished
  if constexpr (AHEAD) { if (has_res) FI_FETCH_RES_PART(0, 0, RV_EARLY) }   // (the wider chains have no registers to spare for it this early)

  f32x16 acc1[NI1];
#pragma unroll
  for (int j = 0; j < NI1; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc1[j][e] = 0.0f;

  {
    // With 64 channels three reduction tiles are in flight in registers: a tile's loads have two multiplies (and
    // whatever the other workgroups of the compute unit do meanwhile) to arrive before they are parked.  The wider
    // chains, whose later phases need every register, keep one.
    constexpr int DEPTH = W1 == 64 ? 3 : 1;
    u32x4 av[DEPTH][4], bw[DEPTH][NI1];
    const int ntiles = d1.Kp / BK;   // Cp is a multiple of 64: every reduction tile lies inside one filter tap
    int kr = 0, ks = 0, kc = kvec;
#define FI_FETCH_1(S, KT)                                                                                    \
    {                                                                                                        \
      const int tvar = ((kr * Wd + ks) * Cp + kc) * 2;                                                       \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                        \
        const bool ok = ((a_rc[i] >> kr) & (a_rc[i] >> (16 + ks)) & 1) != 0;                                 \
        av[S][i] = __builtin_amdgcn_raw_buffer_load_b128(xres, ok ? (uint32_t)(a_row[i] + tvar) : OOB, 0, 0); \
      }                                                                                                      \
      _Pragma("unroll") for (int i = 0; i < NI1; ++i) bw[S][i] = b1_ptr[i][(KT) * (BK / 8)];                 \
      kc += BK;                                                                                              \
      const bool wrap = kc >= Cp;                                                                            \
      kc -= wrap ? Cp : 0;                                                                                   \
      ks += wrap ? 1 : 0;                                                                                    \
      const bool wrap2 = ks == kw;                                                                           \
      ks = wrap2 ? 0 : ks;                                                                                   \
      kr += wrap2 ? 1 : 0;                                                                                   \
    }
#pragma unroll
    for (int u = 0; u < DEPTH; ++u)
      if (u < ntiles) FI_FETCH_1(u, u)
    for (int kt = 0; kt < ntiles; kt += DEPTH) {
#pragma unroll
      for (int u = 0; u < DEPTH; ++u) {
        const int t = kt + u;
        if (t < ntiles) {
#pragma unroll
          for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(&As[(srow + 32 * i) * LDS_STRIDE + kvec]) = av[u][i];
#pragma unroll
          for (int i = 0; i < NI1; ++i) *reinterpret_cast<u32x4*>(&Bs[(srow + 32 * i) * LDS_STRIDE + kvec]) = bw[u][i];
          __syncthreads();
          if (t + DEPTH < ntiles) FI_FETCH_1(u, t + DEPTH)
#pragma unroll
          for (int kk = 0; kk < BK; kk += 16) {
            const int kof = kk + lh * 8;
            const bf16x8 af = *reinterpret_cast<const bf16x8*>(&As[(wave * 32 + lp) * LDS_STRIDE + kof]);
#pragma unroll
            for (int j = 0; j < NI1; ++j) {
              const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(&Bs[(j * 32 + lp) * LDS_STRIDE + kof]);
              acc1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc1[j], 0, 0, 0);
            }
          }
          __syncthreads();
        }
      }
    }
#undef FI_FETCH_1
  }

  if (tid < W1) bias1[tid] = bq1;
#pragma unroll
  for (int i = 0; i < NB2; ++i) bias2[tid + 256 * i] = bq2[i];   // (the table holds MAXN2 entries: rows past B's width are never read)
  if constexpr (N3 > 0) { if (tid < N3) bias3[tid] = bq3; }
  __syncthreads();

  // ---- A's epilogue in registers: bias, activation, one rounding; then into B's operand slots -------------
  uint32_t t1f[W1 / 16][4];
  {
    const Activation<SMOOTH> act1(d1.act);
#pragma unroll
    for (int j = 0; j < NI1; ++j) {
      uint32_t pk[4][2];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b = *reinterpret_cast<const float4*>(bias1 + j * 32 + 8 * g + 4 * lh);
        float v[4] = {acc1[j][4 * g] + b.x, acc1[j][4 * g + 1] + b.y, acc1[j][4 * g + 2] + b.z, acc1[j][4 * g + 3] + b.w};
        act1.apply(v);
        pk[g][0] = pack_bf16x2(v[0], v[1]);
        pk[g][1] = pack_bf16x2(v[2], v[3]);
      }
      uint32_t fr[2][4];
      runs_to_fragments(pk, fr);
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int e = 0; e < 4; ++e) t1f[2 * j + half][e] = fr[half][e];
    }
  }

  // ---- B in chunks of 128 output channels; C accumulates over the chunks (they are its reduction) ----------
  bf16_t* const pt = reinterpret_cast<bf16_t*>(smem) + wave * 32 * PS;   // this wave's patch
  const bool stream_out = (int64_t)M * d2.Cop * 2 > (int64_t)STREAM_OUT_BYTES;
  f32x16 acc3[NI3];
#pragma unroll
  for (int j = 0; j < NI3; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc3[j][e] = 0.0f;
  u32x4 b3v[2][NI3];   // (EARLY) the two tiles of C's weights that a chunk multiplies
  constexpr int WS = 2 * BK + 8;   // (EARLY) row stride of the two tiles parked side by side: 272-byte rows

  for (int c = 0; c < nchunks; ++c) {
    f32x16 acc2[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc2[j][e] = 0.0f;
#pragma unroll
    for (int kt = 0; kt < KT2; ++kt) {
      FI_PARK_B(4)
      __syncthreads();
      if constexpr (EARLY) {   // both tiles of C's weights for this chunk and B's tile for the next: in flight through the epilogue
        _Pragma("unroll") for (int t = 0; t < 2; ++t)
        _Pragma("unroll") for (int i = 0; i < NI3; ++i)
            b3v[t][i] = *reinterpret_cast<const u32x4*>(w3 + (int64_t)(srow + 32 * i) * Kp3 + c * 128 + t * BK + kvec);
        if (c + 1 < nchunks) FI_FETCH_B(w2, W1, (c + 1) * 128, 0, 4)
      } else if (kt + 1 < KT2) FI_FETCH_B(w2, W1, c * 128, (kt + 1) * BK, 4)
      else if (N3 > 0) FI_FETCH_B(w3, Kp3, 0, c * 128, NI3)
      else if (c + 1 < nchunks) FI_FETCH_B(w2, W1, (c + 1) * 128, 0, 4)
      // (memory answers a wave in the order of its requests: the residual rows are asked for after the last weight
      // tile that is parked before they are needed, so that no wait for weights stands behind them)
      if constexpr (!AHEAD) { if (kt == KT2 - 1 && has_res) FI_FETCH_RES_PART(c, 0, RV_EARLY) }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kof = ks * 16 + lh * 8;
        u32x4 au;
#pragma unroll
        for (int e = 0; e < 4; ++e) au[e] = t1f[kt * 4 + ks][e];
        const bf16x8 af = __builtin_bit_cast(bf16x8, au);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(&Bs[(j * 32 + lp) * LDS_STRIDE + kof]);
          acc2[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc2[j], 0, 0, 0);
        }
      }
      __syncthreads();
    }

    // B's epilogue.  The residual rows go through the patch to reach the accumulators' layout; the finished rows go
    // through it the other way to leave as contiguous 16-byte pieces.  The patch belongs to this wave alone.
    const Activation<SMOOTH> act2(d2.act);
    uint32_t t2f[8][4];
    {
      uint32_t pk[4][4][2];
      if constexpr (RV_EARLY < 8) { if (has_res) FI_FETCH_RES_PART(c, RV_EARLY, 8) }
      if (has_res) {
#pragma unroll
        for (int it = 0; it < 8; ++it) *reinterpret_cast<u32x4_a*>(&pt[(prow + 4 * it) * PS + pcol]) = rv[it];
        if constexpr (AHEAD) { if (c + 1 < nchunks) FI_FETCH_RES_PART(c + 1, 0, RV_EARLY) }   // the next chunk's rows travel while this chunk is finished
      }
      wave_lds_fence();
      // Bias, then the residual, then the activation, then the one rounding: the order of the stand-alone kernel.
      // One loop for both cases (two copies of it would meet again with every value of the tile alive twice).  Without a
      // residual the patch holds stale rows: they are read and replaced by -0.0, the one addend that leaves every
      // value, either zero included, as it is.
      uint32_t res_and = has_res ? 0xFFFFFFFFu : 0u, res_or = has_res ? 0u : 0x80008000u;
      asm volatile("" : "+v"(res_and), "+v"(res_or));   // (kept from being turned back into a select per value)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c0 = j * 32 + 8 * g + 4 * lh;
          const float4 b = *reinterpret_cast<const float4*>(bias2 + c * 128 + c0);
          u32x2 r = *reinterpret_cast<const u32x2_a*>(&pt[lp * PS + c0]);
          r[0] = (r[0] & res_and) | res_or;
          r[1] = (r[1] & res_and) | res_or;
          float v[4] = {acc2[j][4 * g] + b.x, acc2[j][4 * g + 1] + b.y, acc2[j][4 * g + 2] + b.z, acc2[j][4 * g + 3] + b.w};
          v[0] += __uint_as_float(r[0] << 16); v[1] += __uint_as_float(r[0] & 0xFFFF0000u);
          v[2] += __uint_as_float(r[1] << 16); v[3] += __uint_as_float(r[1] & 0xFFFF0000u);
          act2.apply(v);
          pk[j][g][0] = pack_bf16x2(v[0], v[1]);
          pk[j][g][1] = pack_bf16x2(v[2], v[3]);
        }
      wave_lds_fence();   // every residual value has been read before the patch is overwritten
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 o;
          o[0] = pk[j][g][0]; o[1] = pk[j][g][1];
          *reinterpret_cast<u32x2_a*>(&pt[lp * PS + j * 32 + 8 * g + 4 * lh]) = o;
        }
      wave_lds_fence();
#pragma unroll
      for (int half = 0; half < 2; ++half) {   // four rows' pieces at a time
        u32x4 orow[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) orow[it] = *reinterpret_cast<const u32x4_a*>(&pt[(prow + 4 * (4 * half + it)) * PS + pcol]);
        if (stream_out) {
#pragma unroll
          for (int it = 0; it < 4; ++it) __builtin_amdgcn_raw_buffer_store_b128(orow[it], y2res, y_off0 + (4 * half + it) * y_step + c * 256, 0, 2);
        } else {
#pragma unroll
          for (int it = 0; it < 4; ++it) __builtin_amdgcn_raw_buffer_store_b128(orow[it], y2res, y_off0 + (4 * half + it) * y_step + c * 256, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      wave_lds_fence();   // the rows have been read before the next chunk's residual lands in the patch
      if constexpr (N3 > 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t fr[2][4];
          runs_to_fragments(pk[j], fr);
#pragma unroll
          for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int e = 0; e < 4; ++e) t2f[2 * j + half][e] = fr[half][e];
        }
      }
    }

    // C: this chunk's 128 channels are reduction elements 128 c .. 128 c + 127 of C
    if constexpr (EARLY) {
      // both tiles side by side in one [N3 x 128] block: one barrier pair, eight reduction steps
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < NI3; ++i) *reinterpret_cast<u32x4*>(&Bs[(srow + 32 * i) * WS + t * BK + kvec]) = b3v[t][i];
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int kof = ks * 16 + lh * 8;
        u32x4 au;
#pragma unroll
        for (int e = 0; e < 4; ++e) au[e] = t2f[ks][e];
        const bf16x8 af = __builtin_bit_cast(bf16x8, au);
#pragma unroll
        for (int j = 0; j < NI3; ++j) {
          const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(&Bs[(j * 32 + lp) * WS + kof]);
          acc3[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc3[j], 0, 0, 0);
        }
      }
      __syncthreads();
    } else if (N3 > 0) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        FI_PARK_B(NI3)
        __syncthreads();
        if (kt == 0) FI_FETCH_B(w3, Kp3, 0, c * 128 + BK, NI3)
        else if (c + 1 < nchunks) FI_FETCH_B(w2, W1, (c + 1) * 128, 0, 4)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int kof = ks * 16 + lh * 8;
          u32x4 au;
#pragma unroll
          for (int e = 0; e < 4; ++e) au[e] = t2f[kt * 4 + ks][e];
          const bf16x8 af = __builtin_bit_cast(bf16x8, au);
#pragma unroll
          for (int j = 0; j < NI3; ++j) {
            const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(&Bs[(j * 32 + lp) * LDS_STRIDE + kof]);
            acc3[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc3[j], 0, 0, 0);
          }
        }
        __syncthreads();
      }
    }
  }
#undef FI_FETCH_B
#undef FI_PARK_B
#undef FI_FETCH_RES
#undef FI_FETCH_RES_PART

  // ---- C's epilogue ---------------------------------------------------------------------------------------
  if constexpr (N3 > 0) {
    const int ys3 = d3.ys;
    const __amdgpu_buffer_rsrc_t y3res = __builtin_amdgcn_make_buffer_rsrc(
        a.abase + d3.y_off, 0, M > 0 ? (int)((((int64_t)M - 1) * ys3 + N3) * 2) : 0, 0x00020000);
    const Activation<SMOOTH> act3(d3.act);
#pragma unroll
    for (int j = 0; j < NI3; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = j * 32 + 8 * g + 4 * lh;
        const float4 b = *reinterpret_cast<const float4*>(bias3 + c0);
        float v[4] = {acc3[j][4 * g] + b.x, acc3[j][4 * g + 1] + b.y, acc3[j][4 * g + 2] + b.z, acc3[j][4 * g + 3] + b.w};
        act3.apply(v);
        u32x2 o;
        o[0] = pack_bf16x2(v[0], v[1]); o[1] = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<u32x2_a*>(&pt[lp * PS + c0]) = o;
      }
    wave_lds_fence();
    constexpr int CPR = NI3 * 4;          // 16-byte pieces per row
    constexpr int NIT = 32 * CPR / 64;    // pieces per lane
    u32x4 orow[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = it * 64 + lane;
      orow[it] = *reinterpret_cast<const u32x4_a*>(&pt[(item / CPR) * PS + (item % CPR) * 8]);
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = it * 64 + lane;
      __builtin_amdgcn_raw_buffer_store_b128(orow[it], y3res, (uint32_t)(((mw + item / CPR) * ys3 + (item % CPR) * 8) * 2), 0, 0);
    }
  }
}

template <typename F>
static int go_chain(F kernel, int blocks, const KArgs& a, hipStream_t s) {
  if (blocks <= 0) return (int)hipSuccess;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

// The launch lists its problems as triples of nodes (A, B, C; a chain of two repeats B in C's place).  The kernel
// has no bounds of its own for what the planner promises, so everything it assumes is checked here first.
int launch_chain(const Launch& L, const KArgs& args, void* stream, const std::vector<Desc>& hd) {
  if (L.n < 3 || L.n % 3 || L.n > FI_MAX_GROUP / 3 * 3 || L.wdtype != FI_BF16 || L.adtype != FI_BF16) return (int)hipErrorInvalidValue;
  const int P = L.n / 3;
  KArgs a = args;
  a.n = P;
  const Desc& f1 = hd[(size_t)L.first_desc];
  const Desc& f3 = hd[(size_t)L.first_desc + 2];
  const int W1 = f1.Co;
  const bool has_c = L.tile != 0;
  const int N3 = has_c ? f3.Co : 0;
  int64_t blocks = 0;
  for (int p = 0; p < P; ++p) {
    const Desc& d1 = hd[(size_t)(L.first_desc + 3 * p)];
    const Desc& d2 = hd[(size_t)(L.first_desc + 3 * p + 1)];
    const Desc& d3 = hd[(size_t)(L.first_desc + 3 * p + 2)];
    a.d[3 * p] = d1; a.d[3 * p + 1] = d2; a.d[3 * p + 2] = d3;
    a.batch[p] = args.batch[3 * p];
    const int b = a.batch[p];
    if (b < 0) return (int)hipErrorInvalidValue;
    // A: dense convolution, bf16 in and out, whole reduction tiles per tap, W1 output channels, unsplit, stored nowhere
    if (d1.Cp % 64 || d1.C != d1.Cp || d1.xs != d1.Cp || d1.Co != W1 || d1.Cop != W1 || (W1 != 64 && W1 != 128) || d1.splits != 1 || d1.ext || d1.out_f32 ||
        d1.pre_kind != 0 || d1.gin > 0 || d1.k < 1 || d1.k > 15 || d1.kw < 1 || d1.kw > 15 || d1.Kp != d1.k * d1.kw * d1.Cp || d1.r_off != kNone ||
        (uint64_t)b * d1.H * d1.W * (uint64_t)d1.Cp * 2 >= (1ull << 31) || (uint64_t)b * d1.Ho * d1.Wo >= (1ull << 24))
      return (int)hipErrorInvalidValue;
    // B: pointwise on A's pixels, W1 -> a multiple of 128 channels
    if (d2.k != 1 || d2.kw != 1 || d2.stride != 1 || d2.pad != 0 || d2.pad_w != 0 || d2.C != W1 || d2.Cp != W1 || d2.Kp != W1 || d2.Co != d2.Cop || d2.Co % 128 ||
        d2.Co < 128 || d2.Co > 1024 || d2.splits != 1 || d2.ext || d2.out_f32 || d2.pre_kind != 0 || d2.gin > 0 || d2.Ho != d1.Ho || d2.Wo != d1.Wo || d2.ys < d2.Cop || d2.y_off == kNone)
      return (int)hipErrorInvalidValue;
    // rows are addressed with 32-bit byte offsets through buffer resources, 127 rows past the last one included
    const uint64_t rows = (uint64_t)b * d1.Ho * d1.Wo + 128;
    if (rows * (uint64_t)d2.ys * 2 >= (1ull << 31) || rows * (uint64_t)d2.Cop * 2 >= (1ull << 31) || (has_c && rows * (uint64_t)d3.ys * 2 >= (1ull << 31)))
      return (int)hipErrorInvalidValue;
    if (has_c) {   // C: pointwise on the same pixels, B's channels -> N3
      if (d3.k != 1 || d3.kw != 1 || d3.stride != 1 || d3.pad != 0 || d3.pad_w != 0 || d3.C != d2.Co || d3.Cp != d2.Co || d3.Kp != d2.Co || d3.Co != N3 ||
          d3.Cop != N3 || (N3 != 64 && N3 != 128) || d3.splits != 1 || d3.ext || d3.out_f32 || d3.pre_kind != 0 || d3.gin > 0 || d3.r_off != kNone ||
          d3.Ho != d1.Ho || d3.Wo != d1.Wo || d3.ys < d3.Cop || d3.y_off == kNone)
        return (int)hipErrorInvalidValue;
    }
    a.first_block[p] = (int32_t)blocks;
    blocks += ((int64_t)b * d1.Ho * d1.Wo + 127) / 128;
    if (blocks > 0x7FFFFFFF) return (int)hipErrorInvalidConfiguration;
  }
  for (int p = P; p <= FI_MAX_GROUP; ++p) a.first_block[p] = (int32_t)blocks;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nb = (int)blocks;
  bool smooth = false;
  for (int p = 0; p < P; ++p)
    for (int t = 0; t < (has_c ? 3 : 2); ++t) smooth = smooth || a.d[3 * p + t].act > FI_ACT_RELU6;
#define FI_CHAIN_CASE(A, C)                                                                          \
  if (W1 == (A) && N3 == (C))                                                                        \
    return smooth ? go_chain(chain_mfma_kernel<A, C, true>, nb, a, s) : go_chain(chain_mfma_kernel<A, C, false>, nb, a, s);
  FI_CHAIN_CASE(64, 0)
  FI_CHAIN_CASE(64, 64)
  FI_CHAIN_CASE(64, 128)
  FI_CHAIN_CASE(128, 0)
  FI_CHAIN_CASE(128, 64)
  FI_CHAIN_CASE(128, 128)
#undef FI_CHAIN_CASE
  return (int)hipErrorInvalidValue;
}

}  // namespace fi
