// Device-side helpers shared by the kernel files: element access, activations, problem lookup, MFMA operand types.
#pragma once

#include <hip/hip_runtime.h>

#include "fi_internal.h"

namespace fi {

// ---------------------------------------------------------------------------------
// element access
// ---------------------------------------------------------------------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round-to-nearest-even (the hardware conversion of gfx950: one instruction for a value, one for a pair)
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }

// ReLU / ReLU6 / identity as branch-free selects (the common case), the smooth activations behind ONE
// block-uniform branch per call, taken around the whole run of values: `act` is the same for every lane of a
// problem, and a caller that hands over everything it holds in one call keeps its epilogue in one basic block.
__device__ __forceinline__ float act_hardswish(float v) { return v * fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) / 6.0f; }
__device__ __forceinline__ float act_hardsigmoid(float v) { return fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) / 6.0f; }
__device__ __forceinline__ float act_sigmoid(float v) { return 1.0f / (1.0f + expf(-v)); }
template <int N>
__device__ __forceinline__ void activate_n(float* v, int act) {
  const int a = __builtin_amdgcn_readfirstlane(act);
  if (a > FI_ACT_RELU6) {
    if (a == FI_ACT_HARDSWISH) {
#pragma unroll
      for (int t = 0; t < N; ++t) v[t] = act_hardswish(v[t]);
    } else if (a == FI_ACT_HARDSIGMOID) {
#pragma unroll
      for (int t = 0; t < N; ++t) v[t] = act_hardsigmoid(v[t]);
    } else if (a == FI_ACT_SILU) {
#pragma unroll
      for (int t = 0; t < N; ++t) v[t] = v[t] * act_sigmoid(v[t]);
    } else {
#pragma unroll
      for (int t = 0; t < N; ++t) v[t] = act_sigmoid(v[t]);
    }
    return;
  }
  const float hi = a == FI_ACT_RELU6 ? 6.0f : INFINITY;
#pragma unroll
  for (int t = 0; t < N; ++t) v[t] = a == FI_ACT_NONE ? v[t] : fminf(fmaxf(v[t], 0.0f), hi);
}
__device__ __forceinline__ float activate(float v, int act) {
  activate_n<1>(&v, act);
  return v;
}

// Finds the problem a workgroup belongs to from the per-launch table of starting workgroup
// indices (kernel arguments: no memory round trip); on return `bid` is the index inside problem `p`.
__device__ __forceinline__ bool find_problem_at(const KArgs& a, int gid, int& p, int& bid) {
  p = 0;
#pragma unroll
  for (int i = 1; i < FI_MAX_GROUP; ++i) p += (i < a.n && gid >= a.first_block[i]) ? 1 : 0;
  bid = gid - a.first_block[p];
  return gid < a.first_block[a.n];
}
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

// The activation of one node, set up once per epilogue and applied to four values at a time.  A kernel variant whose
// launches hold no smooth activation (SMOOTH = false) applies identity / ReLU / ReLU6 in two instructions a value and
// has no branch: a bound that is NaN drops out of max / min (they return the other operand), so identity is
// max(v, NaN), min(., NaN) and ReLU is max(v, 0), min(., NaN): the values activate_n selects, bit for bit.  (The
// bounds pass through an empty asm so that the optimiser, which knows max(v, NaN) = v, does not turn the two
// instructions back into selects.)  The general variant branches once per call.
template <bool SMOOTH>
struct Activation {
  int act;
  float lo, hi;
  __device__ __forceinline__ explicit Activation(int a) : act(a), lo(0.0f), hi(0.0f) {
    if constexpr (!SMOOTH) {
      uint32_t lo_b = a == FI_ACT_NONE ? 0x7FC00000u : 0u, hi_b = a == FI_ACT_RELU6 ? 0x40C00000u : 0x7FC00000u;
      asm volatile("" : "+v"(lo_b), "+v"(hi_b));
      lo = __uint_as_float(lo_b);
      hi = __uint_as_float(hi_b);
    }
  }
  __device__ __forceinline__ void apply(float (&v)[4]) const {
    if constexpr (SMOOTH) {
      activate_n<4>(v, act);
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] = fminf(fmaxf(v[t], lo), hi);
    }
  }
};

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // elements; 144-byte rows keep 16-byte reads conflict-free
constexpr int NXCD = 8;
#ifndef STREAM_OUT_BYTES
#define STREAM_OUT_BYTES (48 << 20)
#endif
constexpr uint32_t OOB = 0x80000000u;  // byte offset past any tensor: the buffer load returns zero

// m / dv for 0 <= m < 2^24 (exact: the float product is off by at most one, then corrected)
__device__ __forceinline__ int fast_div(int m, int dv, float inv) {
  int t = (int)((float)m * inv);
  const int r = m - t * dv;
  t += (r >= dv) ? 1 : 0;
  t -= (r < 0) ? 1 : 0;
  return t;
}

// Which taps of a filter row / column land inside the image, as a bit mask: bit r is set iff 0 <= origin + r < extent
// (r < taps <= 15).  The valid taps are a run, so two shifts replace a loop over the taps.
__device__ __forceinline__ uint32_t taps_inside(int origin, int taps, int extent) {
  const int lo = origin < 0 ? -origin : 0;
  const int hi = extent - origin < taps ? extent - origin : taps;
  return hi > lo ? ((1u << hi) - 1u) & ~((1u << lo) - 1u) : 0u;
}

__device__ __forceinline__ int xcd_contiguous(int bid, int total) {
  const int c = total / NXCD, r = total % NXCD;
  const int x = bid % NXCD, j = bid / NXCD;
  return x * c + (x < r ? x : r) + j;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// From the packed outputs of one 32-channel block (pk[g] = channels 8g + 4h .. + 3 of this lane's pixel, h = lane >> 5,
// as two dwords of bf16 pairs) to the operand fragments of the two 16-element reduction steps the block covers:
// frag[half] = channels 16 half + 8h .. + 7.
__device__ __forceinline__ void runs_to_fragments(const uint32_t (&pk)[4][2], uint32_t (&frag)[2][4]) {
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int dw = 0; dw < 2; ++dw) {
      // lower half keeps its own run g0 and receives the upper half's run g0; the upper half receives the lower
      // half's run g0 + 1 and keeps its own
      const auto r = __builtin_amdgcn_permlane32_swap(pk[2 * half][dw], pk[2 * half + 1][dw], false, false);
      frag[half][dw] = r[0];
      frag[half][2 + dw] = r[1];
    }
}

}  // namespace fi
