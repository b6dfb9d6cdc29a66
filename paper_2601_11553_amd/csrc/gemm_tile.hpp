// Main loop shared by the projection kernels: Y^T tile = W_tile (128 features) x X_tile^T (64 or 128 tokens),
// bf16 (or fp16) operands, fp32 accumulation on the 32x32x16 matrix cores.
//
// A workgroup of 4 wavefronts computes 128 output features x (64 or 128) tokens.  The features are the M side of
// the MFMA and the tokens the N side, so a lane ends up holding 4 consecutive features of one token per accumulator
// quad (8-byte stores into token-major outputs).  Wavefront (wf, wt) owns two 32-feature blocks (fb_lo, fb_hi) --
// chosen by the caller so that features which must meet in the epilogue (a RoPE pair, a gate/up pair) sit in the
// same lane -- and the token blocks wt*NTB .. wt*NTB+NTB-1.  Operand tiles (64 k-elements = 128-byte rows) are
// brought in by direct global->LDS loads into a double-buffered, XOR-swizzled LDS layout (16-byte chunk index
// ^= (row >> 1) & 7: conflict-free reads).
#pragma once

#include "percache_internal.hpp"

namespace pc {
namespace gemm {

constexpr int BK = 64;       // k elements per LDS stage
constexpr int ROW = BK * 2;  // bytes per LDS row
constexpr int BF = 128;      // feature rows per workgroup
constexpr int NW = 4;        // wavefronts per workgroup

template <int NTB>
struct Shape {
  static constexpr int BT = 64 * NTB;  // tokens per workgroup
  static constexpr int W_BYTES = BF * ROW, X_BYTES = BT * ROW, STAGE = W_BYTES + X_BYTES;
  static constexpr int W_INSTR = W_BYTES / 1024 / NW, X_INSTR = X_BYTES / 1024 / NW;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static constexpr int INSTR = W_INSTR + X_INSTR;  // direct-to-LDS load instructions per wavefront and stage
};

__device__ __forceinline__ int swz128(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); }
// s_waitcnt vmcnt(N) alone, N < 64 (expcnt / lgkmcnt fields left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt((N & 0xf) | (7 << 4) | (15 << 8) | (((N >> 4) & 3) << 14));
}

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
  return __builtin_bit_cast(uint2, v);
}
__device__ __forceinline__ void unpack4(uint2 raw, float (&o)[4]) {
  bf16x4 v = __builtin_bit_cast(bf16x4, raw);
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (float)v[e];
}

__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ f32x16 mma(f16x8 a, f16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
template <class T> struct Vec8;
template <> struct Vec8<__bf16> { typedef bf16x8 type; };
template <> struct Vec8<_Float16> { typedef f16x8 type; };

// T: __bf16 or _Float16 (both operands).
// w_row(r): pointer to the first of the K contiguous elements of the weight row that tile row r (0..127) stands
// for (already advanced to the start of the k range when only a slice of the contraction is computed).
// X: token rows of ldx elements, pointing at the first element of the k range; the tile covers token rows
// m0 .. m0 + BT - 1 (clamped to M - 1 when reading); K elements are contracted.
// On return acc[a][t] holds features (a ? fb_hi : fb_lo) * 32 + (r/4)*8 + 4*(lane/32) + r%4 of token
// m0 + (wt*NTB + t)*32 + lane%32 in element r.
// NTW: the weight rows are streamed with the non-temporal policy (use when no other workgroup re-reads them soon).
template <int NTB, bool NTW = false, class T, class WRow>
__device__ __forceinline__ void mainloop(char *lds, WRow w_row, const T *__restrict__ X, int ldx, int m0, int M, int K,
                                         int fb_lo, int fb_hi, f32x16 (&acc)[2][NTB]) {
  using S = Shape<NTB>;
  using V8 = typename Vec8<T>::type;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;

  // direct global -> LDS loads: wavefront instruction i fills bytes [1024 i, 1024 i + 1024) of a tile, lane l
  // the 16 bytes at 1024 i + 16 l, i.e. row (8 i + l / 8), physical chunk l % 8 <- logical chunk (l % 8) ^ swz(row)
  const T *w_src[S::W_INSTR];
  const T *x_src[S::X_INSTR];
#pragma unroll
  for (int k = 0; k < S::W_INSTR; ++k) {
    const int row = (wave + k * NW) * 8 + (lane >> 3);
    w_src[k] = w_row(row) + (((lane & 7) ^ swz128(row)) * 8);
  }
#pragma unroll
  for (int k = 0; k < S::X_INSTR; ++k) {
    const int row = (wave + k * NW) * 8 + (lane >> 3);
    x_src[k] = X + (size_t)min(m0 + row, M - 1) * ldx + (((lane & 7) ^ swz128(row)) * 8);
  }
  auto fetch = [&](int kt, int st) __attribute__((always_inline)) {
    char *base = lds + st * S::STAGE;
#pragma unroll
    for (int k = 0; k < S::W_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(w_src[k] + kt * BK),
                                       (__attribute__((address_space(3))) void *)(base + (wave + k * NW) * 1024), 16, 0, NTW ? 2 : 0);
#pragma unroll
    for (int k = 0; k < S::X_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_src[k] + kt * BK),
                                       (__attribute__((address_space(3))) void *)(base + S::W_BYTES + (wave + k * NW) * 1024), 16, 0, 0);
  };

  // swizzled byte offsets of this lane's operand reads inside its row (row & 31 = l32 for every block)
  int rd[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) rd[ks] = ((2 * ks + g) ^ swz128(l32)) * 16;

#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NTB; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int nk = K / BK;
  fetch(0, 0);
  wait_vmcnt0();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    if (kt + 1 < nk) fetch(kt + 1, st ^ 1);
    const char *wl = lds + st * S::STAGE + (fb_lo * 32 + l32) * ROW;
    const char *wh = lds + st * S::STAGE + (fb_hi * 32 + l32) * ROW;
    const char *xb = lds + st * S::STAGE + S::W_BYTES + ((wt * NTB) * 32 + l32) * ROW;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      V8 a_lo = *(const V8 *)(wl + rd[ks]);
      V8 a_hi = *(const V8 *)(wh + rd[ks]);
#pragma unroll
      for (int t = 0; t < NTB; ++t) {
        V8 b = *(const V8 *)(xb + t * 32 * ROW + rd[ks]);
        acc[0][t] = mma(a_lo, b, acc[0][t]);
        acc[1][t] = mma(a_hi, b, acc[1][t]);
      }
    }
    // the next stage's loads must have landed before anyone reads them; the barrier also retires this stage
    wait_vmcnt0();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
}

// The same main loop for a workgroup of 8 wavefronts on 256 weight rows x 64*NTB tokens: two 128-row halves side by
// side over one token tile, so the token rows are brought in once for twice the features (L2 -> LDS bytes per flop
// drop by a third at NTB = 3).  Wavefront w: half w >> 2, feature blocks (fb_lo, fb_hi) counted over all 8 blocks of
// 32 rows, token group wt.  One workgroup per CU (2 x 56 KB of LDS at NTB = 3).
template <int NTB>
struct WideShape {
  static constexpr int NWV = 8, BFW = 256;
  static constexpr int BT = 64 * NTB;
  static constexpr int W_BYTES = BFW * ROW, X_BYTES = BT * ROW, STAGE = W_BYTES + X_BYTES;
  static constexpr int W_INSTR = W_BYTES / 1024 / NWV, X_INSTR = X_BYTES / 1024 / NWV;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static_assert(W_BYTES % (1024 * NWV) == 0 && X_BYTES % (1024 * NWV) == 0, "whole instructions per wavefront");
};

// One software pipeline over the k-steps: the operands of the next 16 k-elements are read from LDS into a second
// register set while the MFMAs of the current ones run, and the one barrier of a k-step sits before its last quarter.
// There every wavefront has the rest of the current stage in registers, so the stage is requested again (two k-steps
// ahead; the request's instructions go out between the MFMAs of the following quarters, a burst of them would hold
// every wavefront in the issue queue), and the next stage has landed: its first operands are read under the last
// quarter's MFMAs.  Wavefronts 0-3 request the weight rows (8 instructions each), 4-7 the token rows (2 NTB each).
template <int NTB, class T, class WRow>
__device__ __forceinline__ void mainloop_wide(char *lds, WRow w_row, const T *__restrict__ X, int ldx, int m0, int M, int K,
                                              int fb_lo, int fb_hi, int wt, f32x16 (&acc)[2][NTB]) {
  using S = WideShape<NTB>;
  using V8 = typename Vec8<T>::type;
  static_assert(BK == 64, "four quarters of 16 k-elements");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const bool loads_w = wave < 4;
  constexpr int W_PER = S::W_BYTES / 1024 / 4, X_PER = S::X_BYTES / 1024 / 4;  // instructions per wavefront and stage
  static_assert(W_PER == 8 && X_PER <= 8 && X_PER >= 4, "request split below");
  const T *src[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int row = ((wave & 3) * (loads_w ? W_PER : X_PER) + (k < (loads_w ? W_PER : X_PER) ? k : 0)) * 8 + (lane >> 3);
    src[k] = (loads_w ? w_row(row) : X + (size_t)min(m0 + row, M - 1) * ldx) + (((lane & 7) ^ swz128(row)) * 8);
  }
  char *const dst = lds + (loads_w ? 0 : S::W_BYTES) + (wave & 3) * (loads_w ? W_PER : X_PER) * 1024;
  const int nk = K / BK;
  int f_kt = 0;  // the k-step the next request brings (past the last one: the last one again, into a stage nobody reads)
  // instructions k0 .. k1 - 1 of that request (a token wavefront has fewer: the surplus is skipped)
  auto request_part = [&](int st, int k0, int k1) __attribute__((always_inline)) {
    if (loads_w) {
#pragma unroll
      for (int k = k0; k < k1; ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[k] + f_kt * BK),
                                         (__attribute__((address_space(3))) void *)(dst + st * S::STAGE + k * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int k = k0; k < (k1 < X_PER ? k1 : X_PER); ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[k] + f_kt * BK),
                                         (__attribute__((address_space(3))) void *)(dst + st * S::STAGE + k * 1024), 16, 0, 0);
    }
  };
  auto advance = [&]() __attribute__((always_inline)) { f_kt = f_kt + 1 < nk ? f_kt + 1 : f_kt; };

  int rd[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) rd[q] = ((2 * q + g) ^ swz128(l32)) * 16;
  const int lo_off = (fb_lo * 32 + l32) * ROW, hi_off = (fb_hi * 32 + l32) * ROW, x_off = S::W_BYTES + ((wt * NTB) * 32 + l32) * ROW;
  V8 oa[2][2], ob[2][NTB];  // two register sets
  auto read_ops = [&](int set, int st, int q) __attribute__((always_inline)) {
    const char *base = lds + st * S::STAGE + rd[q];
    oa[set][0] = *(const V8 *)(base + lo_off);
    oa[set][1] = *(const V8 *)(base + hi_off);
#pragma unroll
    for (int t = 0; t < NTB; ++t) ob[set][t] = *(const V8 *)(base + x_off + t * 32 * ROW);
  };
  auto mma_ops = [&](int set) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < NTB; ++t) {
      acc[0][t] = mma(oa[set][0], ob[set][t], acc[0][t]);
      acc[1][t] = mma(oa[set][1], ob[set][t], acc[1][t]);
    }
  };
  // one MFMA, one LDS read, ... and `loads` request instructions among them
  auto interleave = [&](int loads) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NTB + 2; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if ((i & 1) == 0 && i / 2 < loads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * NTB - (NTB + 2), 0);
  };
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NTB; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  request_part(0, 0, 8);
  advance();
  wait_vmcnt0();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  request_part(1, 0, 3);  // (the rest of it under the first two quarters below)
  read_ops(0, 0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    request_part(st ^ 1, 3, 6);
    read_ops(1, st, 1);
    mma_ops(0);
    interleave(3);
    request_part(st ^ 1, 6, 8);
    read_ops(0, st, 2);
    mma_ops(1);
    interleave(2);
    advance();
    read_ops(1, st, 3);
    mma_ops(0);
    interleave(0);
    // every read of this stage is in registers and this wavefront's part of the next stage has landed
    __builtin_amdgcn_s_waitcnt(7 << 4);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    request_part(st, 0, 3);    // k-step kt + 2
    read_ops(0, st ^ 1, 0);    // (past the last k-step: whatever the other stage holds, never multiplied)
    mma_ops(1);
    interleave(3);
  }
  wait_vmcnt0();  // (the surplus request of the last k-steps)
  __builtin_amdgcn_s_barrier();
}

// The same contraction for workgroups that own only a few k-steps (a slice of a split contraction): NS LDS stages,
// all of them requested before the first MFMA, so that a workgroup with up to NS k-steps pays one memory latency
// instead of one per step.  A stage is refilled (k-step kt + NS) once every wavefront has finished reading it.
// Arguments and result as for mainloop(); the LDS buffer holds NS * Shape<NTB>::STAGE bytes.
template <int NTB, bool NTW, int NS, class T, class WRow>
__device__ __forceinline__ void mainloop_deep(char *lds, WRow w_row, const T *__restrict__ X, int ldx, int m0, int M,
                                              int K, int fb_lo, int fb_hi, f32x16 (&acc)[2][NTB]) {
  using S = Shape<NTB>;
  using V8 = typename Vec8<T>::type;
  static_assert(NS >= 2 && NS <= 4 && (NS - 1) * S::INSTR < 64, "stage count");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;
  const T *w_src[S::W_INSTR];
  const T *x_src[S::X_INSTR];
#pragma unroll
  for (int k = 0; k < S::W_INSTR; ++k) {
    const int row = (wave + k * NW) * 8 + (lane >> 3);
    w_src[k] = w_row(row) + (((lane & 7) ^ swz128(row)) * 8);
  }
#pragma unroll
  for (int k = 0; k < S::X_INSTR; ++k) {
    const int row = (wave + k * NW) * 8 + (lane >> 3);
    x_src[k] = X + (size_t)min(m0 + row, M - 1) * ldx + (((lane & 7) ^ swz128(row)) * 8);
  }
  auto fetch = [&](int kt, int st) __attribute__((always_inline)) {
    char *base = lds + st * S::STAGE;
#pragma unroll
    for (int k = 0; k < S::W_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(w_src[k] + kt * BK),
                                       (__attribute__((address_space(3))) void *)(base + (wave + k * NW) * 1024), 16, 0, NTW ? 2 : 0);
#pragma unroll
    for (int k = 0; k < S::X_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_src[k] + kt * BK),
                                       (__attribute__((address_space(3))) void *)(base + S::W_BYTES + (wave + k * NW) * 1024), 16, 0, 0);
  };
  int rd[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) rd[ks] = ((2 * ks + g) ^ swz128(l32)) * 16;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NTB; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < NS; ++s)
    if (s < nk) fetch(s, s);
  int st = 0;
  for (int kt = 0; kt < nk; ++kt) {
    // k-step kt has landed once at most the loads of the (up to NS - 1) later steps in flight are outstanding
    const int later = min(NS - 1, nk - 1 - kt);
    if (later >= 3) wait_vmcnt<(NS > 3 ? 3 : 0) * S::INSTR>();
    else if (later == 2) wait_vmcnt<(NS > 2 ? 2 : 0) * S::INSTR>();
    else if (later == 1) wait_vmcnt<S::INSTR>();
    else wait_vmcnt0();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const char *wl = lds + st * S::STAGE + (fb_lo * 32 + l32) * ROW;
    const char *wh = lds + st * S::STAGE + (fb_hi * 32 + l32) * ROW;
    const char *xb = lds + st * S::STAGE + S::W_BYTES + ((wt * NTB) * 32 + l32) * ROW;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      V8 a_lo = *(const V8 *)(wl + rd[ks]);
      V8 a_hi = *(const V8 *)(wh + rd[ks]);
#pragma unroll
      for (int t = 0; t < NTB; ++t) {
        V8 b = *(const V8 *)(xb + t * 32 * ROW + rd[ks]);
        acc[0][t] = mma(a_lo, b, acc[0][t]);
        acc[1][t] = mma(a_hi, b, acc[1][t]);
      }
    }
    if (kt + NS < nk) {
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();  // every wavefront has read this stage
      asm volatile("" ::: "memory");
      fetch(kt + NS, st);
    }
    st = st + 1 == NS ? 0 : st + 1;
  }
}

// Few token rows, many output features: the weight stream bounds the projection, and it takes many workgroups to pull
// it.  Here a workgroup owns only 32 weight rows -- N/32 workgroups -- and up to 128 token rows over the WHOLE
// contraction (no slices to add up afterwards); wavefront w owns token block w.  NS stages of 64 k-elements
// (4 KB of weights + 16 KB of tokens each), NS - 1 of them in flight, one barrier per k-step.
//   w_row(r): the K contiguous elements of the weight row that tile row r (0..31) stands for.
//   On return acc[r] = tile row (r/4)*8 + 4*(lane/32) + r%4 of token m0 + 32*wave + lane%32.
struct Skinny {
  static constexpr int W_BYTES = 32 * ROW, X_BYTES = 128 * ROW, STAGE = W_BYTES + X_BYTES;
  static constexpr int INSTR = 1 + X_BYTES / 1024 / NW;  // direct-to-LDS load instructions per wavefront and stage
};
template <int NS, class T, class WRow>
__device__ __forceinline__ void mainloop_skinny(char *lds, WRow w_row, const T *__restrict__ X, int ldx, int m0, int M, int K,
                                                f32x16 &acc) {
  using S = Skinny;
  using V8 = typename Vec8<T>::type;
  static_assert(NS >= 2 && NS <= 7 && (NS - 1) * S::INSTR < 64, "stage count");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  constexpr int XI = S::X_BYTES / 1024 / NW;
  const T *w_src;
  const T *x_src[XI];
  {
    const int row = wave * 8 + (lane >> 3);  // the 32 weight rows: one load instruction per wavefront
    w_src = w_row(row) + (((lane & 7) ^ swz128(row)) * 8);
  }
#pragma unroll
  for (int k = 0; k < XI; ++k) {
    const int row = (wave + k * NW) * 8 + (lane >> 3);
    x_src[k] = X + (size_t)min(m0 + row, M - 1) * ldx + (((lane & 7) ^ swz128(row)) * 8);
  }
  const int nk = K / BK;
  auto fetch = [&](int kt, int st) __attribute__((always_inline)) {
    char *base = lds + st * S::STAGE;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(w_src + kt * BK),
                                     (__attribute__((address_space(3))) void *)(base + wave * 1024), 16, 0, 2);
#pragma unroll
    for (int k = 0; k < XI; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_src[k] + kt * BK),
                                       (__attribute__((address_space(3))) void *)(base + S::W_BYTES + (wave + k * NW) * 1024), 16, 0, 0);
  };
  int rd[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) rd[ks] = ((2 * ks + g) ^ swz128(l32)) * 16;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  // two accumulation chains (even / odd k-steps of 16): a lone chain would wait out every MFMA's latency
  f32x16 acc_odd;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc_odd[r] = 0.f;

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk) fetch(s, s);
  int st = 0, fill = NS - 1;  // stage of k-step kt; stage that k-step kt + NS - 1 goes to (the one kt - 1 has left)
  for (int kt = 0; kt < nk; ++kt) {
    const int later = min(NS - 2, nk - 1 - kt);  // k-steps in flight behind this one
    if (later >= 5) wait_vmcnt<(NS > 6 ? 5 : 0) * S::INSTR>();
    else if (later == 4) wait_vmcnt<(NS > 5 ? 4 : 0) * S::INSTR>();
    else if (later == 3) wait_vmcnt<(NS > 4 ? 3 : 0) * S::INSTR>();
    else if (later == 2) wait_vmcnt<(NS > 3 ? 2 : 0) * S::INSTR>();
    else if (later == 1) wait_vmcnt<(NS > 2 ? 1 : 0) * S::INSTR>();
    else wait_vmcnt0();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();  // k-step kt has landed for everyone, and everyone has left the stage of kt - 1
    asm volatile("" ::: "memory");
    if (kt + NS - 1 < nk) fetch(kt + NS - 1, fill);
    const char *wb = lds + st * S::STAGE + l32 * ROW;
    const char *xb = lds + st * S::STAGE + S::W_BYTES + (wave * 32 + l32) * ROW;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const V8 a = *(const V8 *)(wb + rd[ks]);
      const V8 b = *(const V8 *)(xb + rd[ks]);
      if (ks & 1) acc_odd = mma(a, b, acc_odd); else acc = mma(a, b, acc);
    }
    st = st + 1 == NS ? 0 : st + 1;
    fill = fill + 1 == NS ? 0 : fill + 1;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] += acc_odd[r];
}

}  // namespace gemm
}  // namespace pc
