// gfx950 kernel of the quantized Adam step: the per-layer loop body of Algorithm 1 of the paper
// (moment update, Quantize(m,'linear'), Quantize(v,'log'), bias correction of the quantized
// moments, decoupled-weight-decay update) with the block quantizers of Section 3.5 and the
// per-layer statistics of Section 3.3, fused into one pass over HBM.
//
// Arithmetic contract: IEEE binary32, every operation rounded on its own (build with
// -ffp-contract=off); division and square root are the correctly rounded ones.
//
// Work decomposition: one wavefront owns one 2048-element tile at a time and processes it as four
// quarters of 2 rows: a quarter's working set fits the 80 registers of six waves per SIMD with
// nothing spilled to scratch memory, so the kernel's HBM traffic is the algorithmic traffic.
// In row i lane j holds the 4 elements 256*i + 4*j + e, so
// every parameter and gradient access is a coalesced 16-byte (8-byte for bf16) per-lane access,
// and a block of K = 64/128/256 consecutive elements is 16/32/64 neighbouring lanes of one row.
// The lane's 32 codes of a state are exactly b 32-bit words; word p of all lanes is one contiguous
// 256-byte row of the code buffer.  A quarter reads the words that hold its 8 codes and writes
// the words it completes; the bits of a word shared with the next quarter travel in a register.
//
// Only the bit-stream unpack and pack are specialised per width (small switch arms); all
// arithmetic is width-generic and takes the width through table offsets and constants.
#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "stq_device.h"
#include "stq_tables.h"

#pragma clang fp contract(off)

namespace stq {
namespace {

constexpr int XS = 68;  // row stride (words) of the transpose scratch: keeps 16-byte alignment, shifts banks
// per-wave LDS scratch: XR[4][XS] partial maxima (later the den table), old scales, new scales, reciprocals
constexpr int kWaveScratch = 4 * XS + 3 * 64;
constexpr int kLdsWords = kTabWords + kWavesPerGroup * kWaveScratch;  // + the statistics slices in that variant
constexpr int kStatFlushTiles = 16;  // fp32 lane sums are widened to fp64 every this many tiles
constexpr uint32_t kDenEntries = 128;  // capacity of the per-wave den table (8 bytes per entry, inside XR)

// Pointers that arrive through the tensor table are loaded from memory, so the compiler cannot
// see that they are global; say so, to get global_load/global_store instead of flat accesses.
#define STQ_GLOBAL __attribute__((address_space(1)))
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <class T>
__device__ __forceinline__ STQ_GLOBAL T* as_global(T* p) { return (STQ_GLOBAL T*)p; }

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// value at byte offset `off` of an LDS float table
__device__ __forceinline__ float lds_at(const float* base, uint32_t off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + off);
}

__device__ __forceinline__ void wave_lds_sync() {
  // LDS operations of one wavefront execute in order; this only stops the compiler from moving
  // accesses of other lanes' data across the point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------- bit streams
// Within a quarter, code n (0..7) of width B sits at bits [n*B, n*B+B) of the quarter's local stream
// (at most 64 bits, words w[0], w[1]).
// Bits [SH, SH+B) of x in one instruction.  Written as the instruction itself: from the plain expression
// the compiler makes a shift and a mask, and then cannot fold the table offset that follows into either.
template <int SH, int B>
__device__ __forceinline__ uint32_t bit_field(uint32_t x) {
  uint32_t r;
  asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "n"(SH), "n"(B));
  return r;
}

template <int B, int N>
__device__ __forceinline__ uint32_t extract(const uint32_t (&w)[3]) {
  constexpr int off = N * B, p = off >> 5, sh = off & 31;
  if (sh + B <= 32) return bit_field<sh, B>(w[p]);
  // a code that straddles two words: align it first
  return bit_field<0, B>(__builtin_amdgcn_alignbit(w[p + 1], w[p], static_cast<uint32_t>(sh)));
}

template <int B>
__device__ __forceinline__ void insert(uint32_t (&w)[3], int n, uint32_t code) {
  const int off = n * B, p = off >> 5, sh = off & 31;
  if (sh == 0) w[p] = code; else w[p] |= code << sh;
  if (sh + B > 32) w[p + 1] = code >> (32 - sh);  // first bits of the next word
}

// The 8 codes of a quarter as byte offsets into the width's value table: (code << 2) | (4 << B).
// lw holds the lane's words from the one that contains the quarter's first bit; s0 (0, 8, 16 or
// 24) is the position of that bit in lw[0].
template <int B>
__device__ __forceinline__ void unpack_offsets(const uint32_t* lw, uint32_t s0, uint32_t (&off)[8]) {
  uint32_t w[3];
  w[0] = __builtin_amdgcn_alignbit(lw[1], lw[0], s0);
  w[1] = __builtin_amdgcn_alignbit(lw[2], lw[1], s0);
  w[2] = 0u;
  off[0] = (extract<B, 0>(w) << 2) | (4u << B);
  off[1] = (extract<B, 1>(w) << 2) | (4u << B);
  off[2] = (extract<B, 2>(w) << 2) | (4u << B);
  off[3] = (extract<B, 3>(w) << 2) | (4u << B);
  off[4] = (extract<B, 4>(w) << 2) | (4u << B);
  off[5] = (extract<B, 5>(w) << 2) | (4u << B);
  off[6] = (extract<B, 6>(w) << 2) | (4u << B);
  off[7] = (extract<B, 7>(w) << 2) | (4u << B);
}

// Pack the 8 codes of a quarter behind the s0 bits that `carry` holds of the current word, store
// the words this completes (at C, word stride 64) and keep the rest in `carry`.
template <int B>
__device__ __forceinline__ void pack_store(const uint32_t (&code)[8], STQ_GLOBAL uint32_t* C, uint32_t s0,
                                           uint32_t& carry, uint32_t lane) {
  uint32_t ow[3] = {0u, 0u, 0u};
#pragma unroll
  for (int n = 0; n < 8; ++n) insert<B>(ow, n, code[n]);
  const unsigned long long x = (static_cast<unsigned long long>(ow[1]) << 32) | ow[0];
  const unsigned long long lo = x << s0;
  const uint32_t m0 = carry | static_cast<uint32_t>(lo);
  const uint32_t m1 = static_cast<uint32_t>(lo >> 32);
  const uint32_t m2 = s0 ? (ow[1] >> (32u - s0)) : 0u;
  const uint32_t done = (s0 + 8u * B) >> 5;  // complete words: 0, 1 or 2
  if (done >= 1) C[lane] = m0;
  if (done >= 2) C[64u + lane] = m1;
  carry = done == 0 ? m0 : (done == 1 ? m1 : m2);
}

#define STQ_SWITCH_BITS(bits, CALL)               \
  switch (bits) {                                 \
    case 2: { constexpr int B = 2; CALL; } break; \
    case 3: { constexpr int B = 3; CALL; } break; \
    case 4: { constexpr int B = 4; CALL; } break; \
    case 5: { constexpr int B = 5; CALL; } break; \
    case 6: { constexpr int B = 6; CALL; } break; \
    case 7: { constexpr int B = 7; CALL; } break; \
    default: { constexpr int B = 8; CALL; } break; \
  }

// element n (0..7) of this lane in quarter q is real (not pad) in a tile with n_valid elements
__device__ __forceinline__ bool is_valid(int n, uint32_t q, int lane, uint32_t n_valid) {
  return (512u * q + static_cast<uint32_t>(256 * (n >> 2) + 4 * lane + (n & 3))) < n_valid;
}

// x from the lane that a DPP control word names (all lanes of the wave active)
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each row of 16 lanes

// -------------------------------------------------------------------- statistics
// (The sums of squares use fused multiply-adds: the fixed operation order binds the Adam
// arithmetic, not the statistics, which are compared within a tolerance.)
// Running statistics of one wave, kept in its LDS slice so that they cost no registers between the places
// that add to them.  A contribution is first combined over a few neighbouring lanes with DPP steps, then one
// lane of the group adds it to the group's word with an LDS atomic that returns nothing: the wave does not
// wait for it, where a read-modify-write would put an LDS round trip into every quarter's dependency chain
// (that latency, not the arithmetic, was most of the statistics' cost: it showed when fewer waves were
// resident to hide it).  The atomics are issued from 8 or 16 lanes: from all 64 they are several times slower.
//  * The gradient's three sums (all that the bit-width decision reads, Eq. 2, 3, 8) are taken in fp64 from the
//    first addition on: fp64 vector additions issue at the rate of fp32 ones here, and a decision that compares a
//    score with a threshold should not hinge on the rounding of a sum (the variance in Eq. 3 is a difference of
//    two such sums).  Groups of four lanes, 16-word slots; the gradient's maximum likewise in a 16-word slot of
//    bit patterns (all maxima are non-negative, so they order like their bit patterns).
//  * S = 1 adds the moments' six fp32 sums (groups of eight lanes, 8-word slots) and two maxima (the owner lanes
//    of the block scales hold them: lanes 0..31 the first moment's, 32..63 the second's, so a group of four is
//    of one kind); the sums since the last widening are added to fp64 totals (lane k < 6 of the last slot)
//    every kStatFlushTiles tiles.
// S = 2: the gradient's statistics only; the slice stays small enough for three workgroups per CU.
enum GradSlot { kLGSum = 0, kLGAbs, kLGSq };
enum MomentSlot { kLMSum = 0, kLMSq, kLMErr, kLVSum, kLVSq, kLVErr };

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  const uint64_t u = __builtin_bit_cast(uint64_t, x);
  const uint64_t lo = dpp_u32<CTRL>(static_cast<uint32_t>(u)), hi = dpp_u32<CTRL>(static_cast<uint32_t>(u >> 32));
  return __builtin_bit_cast(double, (hi << 32) | lo);
}
// Sums and maxima over groups of 4, 8 or 16 neighbouring lanes, left in every lane of the group.  DPP steps
// only: a shuffle through LDS needs a lane-dependent address register, and the compiler keeps those
// alive across the whole tile loop.
__device__ __forceinline__ double quad_sum(double x) {
  x += dpp_f64<kDppXor1>(x);
  x += dpp_f64<kDppXor2>(x);
  return x;
}
__device__ __forceinline__ double octet_sum(double x) {
  x = quad_sum(x);
  x += dpp_f64<kDppHalfMirror>(x);
  return x;
}
__device__ __forceinline__ double row_sum(double x) {
  x = octet_sum(x);
  x += dpp_f64<kDppMirror>(x);
  return x;
}
__device__ __forceinline__ float octet_sum(float x) {
  x += u2f(dpp_u32<kDppXor1>(f2u(x)));
  x += u2f(dpp_u32<kDppXor2>(f2u(x)));
  x += u2f(dpp_u32<kDppHalfMirror>(f2u(x)));
  return x;
}
__device__ __forceinline__ uint32_t quad_max(uint32_t x) {
  x = max(x, dpp_u32<kDppXor1>(x));
  x = max(x, dpp_u32<kDppXor2>(x));
  return x;
}
__device__ __forceinline__ uint32_t octet_max(uint32_t x) {
  x = quad_max(x);
  return max(x, dpp_u32<kDppHalfMirror>(x));
}
__device__ __forceinline__ uint32_t row_max(uint32_t x) {
  x = octet_max(x);
  return max(x, dpp_u32<kDppMirror>(x));
}

// Layout of a wave's slice (32-bit words), S = 2 | S = 1:
//   gradient sums  3 slots of G doubles, G = 16 | 8 (one word per group of 64/G lanes)
//   maxima         16 | 32 words: [0, G) max|g|; S = 1: [16, 24) max|m| (lanes 0..31 own the first moment's
//                  block scales), [24, 32) max v (lanes 32..63); words [8, 16) stay 0
//   S = 1 only     moment sums: 6 slots of 8 floats; fp64 totals of the six since the last flush (+ pad)
// S = 1 takes the smaller gradient slots so that three workgroups still fit a CU's LDS.
template <int S>
struct LaneStats {
  static constexpr int kGShift = S == 1 ? 3 : 2;  // log2 of the lanes that share a gradient word
  static constexpr int kG = 64 >> kGShift;        // words per gradient slot
  static constexpr int kMaxWords = S == 1 ? 32 : 16;
  static constexpr int kMomentSums = S == 1 ? 6 : 0;
  static constexpr int kMaxOff = 3 * 2 * kG, kMomentOff = kMaxOff + kMaxWords, kWideOff = kMomentOff + 6 * 8;
  static constexpr int kWords = S == 0 ? 0 : (S == 1 ? kWideOff + 2 * 6 + 4 : kMomentOff);
  float* acc;      // this wave's slice, null in the plain kernel
  uint32_t tiles;  // tiles since the last widening (uniform; stripes only)
  __device__ __forceinline__ double* grad_sums() const { return reinterpret_cast<double*>(acc); }
  __device__ __forceinline__ uint32_t* maxima() const { return reinterpret_cast<uint32_t*>(acc) + kMaxOff; }
  __device__ __forceinline__ float* moment_sums() const { return acc + kMomentOff; }
  __device__ __forceinline__ double& wide(int k) const { return reinterpret_cast<double*>(acc + kWideOff)[k]; }

  __device__ __forceinline__ void add_grad(int k, int lane, double x) {
    x = S == 1 ? octet_sum(x) : quad_sum(x);
    if ((lane & ((1 << kGShift) - 1)) == 0)
      __hip_atomic_fetch_add(&grad_sums()[k * kG + (lane >> kGShift)], x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  }
  __device__ __forceinline__ void max_grad(int lane, float x) {
    const uint32_t xb = S == 1 ? octet_max(f2u(x)) : quad_max(f2u(x));
    if ((lane & ((1 << kGShift) - 1)) == 0)
      __hip_atomic_fetch_max(maxima() + (lane >> kGShift), xb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  }
  __device__ __forceinline__ void add(int slot, int lane, float x) {
    x = octet_sum(x);
    if ((lane & 7) == 0)
      __hip_atomic_fetch_add(&moment_sums()[slot * 8 + (lane >> 3)], x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  }
  // the maximum of a block of a moment, from its owner lanes (a quad is of one kind: see the layout)
  __device__ __forceinline__ void max_moment(int lane, float x) {
    const uint32_t xb = quad_max(f2u(x));
    if ((lane & 3) == 0)
      __hip_atomic_fetch_max(maxima() + 16 + (lane >> 2), xb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  }
  __device__ __forceinline__ void clear_moment_sums(int lane) {
    if (S == 1 && lane < 48) moment_sums()[lane] = 0.0f;
    tiles = 0;
  }
  __device__ __forceinline__ void clear_grad(int lane) {
    if (lane < 3 * kG) grad_sums()[lane] = 0.0;
    if (lane < kMaxWords) maxima()[lane] = 0u;
  }
  __device__ __forceinline__ void clear_all(int lane) {
    clear_grad(lane);
    if (S == 1) {
      clear_moment_sums(lane);
      if (lane < 6) wide(lane) = 0.0;
    }
  }
  // The reductions of a slice, for the flushes below (call wave_lds_sync() first).
  // Gradient sum k (0..2), complete, in the lanes [k*kG, (k+1)*kG); zero in the lanes from 3*kG on.
  __device__ __forceinline__ double reduced_grad(int lane) const {
    const double x = lane < 3 * kG ? grad_sums()[lane] : 0.0;
    return S == 1 ? octet_sum(x) : row_sum(x);
  }
  // Moment sum k (0..5) since the last clearing, in the lanes [8k, 8k+8); zero from lane 48 on.
  __device__ __forceinline__ double reduced_moment(int lane) const {
    return octet_sum(lane < 48 ? static_cast<double>(moment_sums()[lane]) : 0.0);
  }
  // max|g| in lane 0; S = 1: max|m| in lane 16, max v in lane 24.
  __device__ __forceinline__ uint32_t reduced_max(int lane) const {
    const uint32_t x = lane < kMaxWords ? maxima()[lane] : 0u;
    return S == 1 ? octet_max(x) : row_max(x);
  }
  // lane holds gradient sum `k` / moment sum `k` / maximum `k` (0 g, 1 m, 2 v) of the reductions above
  __device__ __forceinline__ static bool grad_lead(int lane, int& k) { k = lane >> (6 - kGShift); return lane < 3 * kG && (lane & (kG - 1)) == 0; }
  __device__ __forceinline__ static bool moment_lead(int lane, int& k) { k = lane >> 3; return S == 1 && lane < 48 && (lane & 7) == 0; }
  __device__ __forceinline__ static bool max_lead(int lane, int& k) {
    k = lane == 0 ? 0 : (lane == 16 ? 1 : 2);
    return lane == 0 || (S == 1 && (lane == 16 || lane == 24));
  }
};

// S = 1: the moments' fp32 sums -> the wave's fp64 totals
template <int S>
__device__ __forceinline__ void widen_stats(LaneStats<S>& s, int lane) {
  if (S != 1) return;
  asm volatile("" : "+v"(lane));  // nothing derived from the lane index is worth keeping across the tile loop
  wave_lds_sync();                // the atomics of every lane before the reads below
  const double t = s.reduced_moment(lane);
  int k;
  if (LaneStats<S>::moment_lead(lane, k)) s.wide(k) += t;
  s.clear_moment_sums(lane);
}

// the wave's statistics -> the tensor's global slots; the slice is cleared  (stripes)
template <int S>
__device__ __forceinline__ void flush_stats(LaneStats<S>& s, double* slot, int lane) {
  asm volatile("" : "+v"(lane));
  wave_lds_sync();
  const double g = s.reduced_grad(lane);
  const uint32_t mx = s.reduced_max(lane);
  uint32_t* out = reinterpret_cast<uint32_t*>(&slot[kMaxGM]);  // max |g|, max |m|, max v: consecutive words
  int k;
  if (LaneStats<S>::grad_lead(lane, k)) atomicAdd(&slot[kGSum + k], g);
  if (LaneStats<S>::max_lead(lane, k)) atomicMax(&out[k], mx);
  if (S == 1) {
    widen_stats(s, lane);
    wave_lds_sync();
    if (lane < 6) atomicAdd(&slot[kMSum + lane], s.wide(lane));
  }
  s.clear_all(lane);
}

// ---- statistics under the ticket schedule ----
// A wave changes tensor with almost every tile there, so it cannot keep sums per tensor.  Instead, after every
// tile, the wave reduces its values over its lanes, clears its slice and leaves the values in its record of
// the current ticket in LDS.  After the ticket's barrier wave 0 adds up the records of the workgroup's waves
// and adds the result to the tensor's global slots: one set of global atomics per workgroup and ticket.  The
// records belong to the tensor of the ticket's first unit; a wave whose tile lies in another tensor (a ticket
// that straddles a tensor boundary) adds to that tensor's global slots itself and leaves an empty record.
template <int S>
struct TicketRecord {
  double sum[S == 1 ? 9 : 3];           // in the order of the global slots from kGSum on
  uint32_t max_bits[S == 1 ? 4 : 2];    // max|g|, (max|m|, max v,) pad
};

// after a tile: the wave's values -> its record (or, for a straddling tile, the tensor's global slots)
template <int S>
__device__ __forceinline__ void ticket_stats_tile(LaneStats<S>& s, TicketRecord<S>* rec, bool in_wg_tensor, double* slot, int lane) {
  asm volatile("" : "+v"(lane));
  wave_lds_sync();
  double g = s.reduced_grad(lane);
  double mo = S == 1 ? s.reduced_moment(lane) : 0.0;
  uint32_t mx = s.reduced_max(lane);
  s.clear_grad(lane);
  s.clear_moment_sums(lane);
  int kg, km, kx;
  const bool lg = LaneStats<S>::grad_lead(lane, kg), lm = LaneStats<S>::moment_lead(lane, km), lx = LaneStats<S>::max_lead(lane, kx);
  if (!in_wg_tensor) {
    if (lg) atomicAdd(&slot[kGSum + kg], g);
    if (lm) atomicAdd(&slot[kMSum + km], mo);
    if (lx) atomicMax(reinterpret_cast<uint32_t*>(&slot[kMaxGM]) + kx, mx);
    g = 0.0;
    mo = 0.0;
    mx = 0u;
  }
  if (lg) rec->sum[kg] = g;
  if (lm) rec->sum[3 + km] = mo;
  if (lx) rec->max_bits[kx] = mx;
}

// wave 0, after the ticket's barrier: the records of the workgroup's waves -> the tensor's global slots
template <int S>
__device__ __forceinline__ void ticket_stats_flush(const TicketRecord<S>* recs, double* slot, int lane) {
  static_assert(kWavesPerGroup == 8, "lane 8k + w takes value k of wave w's record");
  asm volatile("" : "+v"(lane));
  constexpr int kSums = S == 1 ? 9 : 3, kMaxima = S == 1 ? 3 : 1;
  const TicketRecord<S>& r = recs[lane & 7];
  const int k = lane >> 3;
  const double x = octet_sum(k < kSums ? r.sum[k] : 0.0);  // sums 0..7
  if ((lane & 7) == 0 && k < kSums) atomicAdd(&slot[kGSum + k], x);
  if (S == 1) {
    const double y = octet_sum(lane < 8 ? r.sum[kSums - 1] : 0.0);  // the ninth
    if (lane == 0) atomicAdd(&slot[kGSum + 8], y);
  }
  const uint32_t mx = octet_max(k < kMaxima ? r.max_bits[k] : 0u);
  if ((lane & 7) == 0 && k < kMaxima) atomicMax(reinterpret_cast<uint32_t*>(&slot[kMaxGM]) + k, mx);
}

// Correctly rounded square root for x = 0 or 2^-96 <= x <= 2^96: the hardware estimate is within
// one ulp; the residuals x - next_down*s and x - next_up*s (exact in an fma) tell which of the
// three neighbours is the rounded root.  This is the IEEE expansion without its input scaling.
__device__ __forceinline__ float sqrt_rn_safe(float x) {
  float s = __builtin_amdgcn_sqrtf(x);
  const float s_dn = u2f(f2u(s) - 1u), s_up = u2f(f2u(s) + 1u);
  const float t_dn = __builtin_fmaf(-s_dn, s, x);
  const float t_up = __builtin_fmaf(-s_up, s, x);
  s = (t_dn <= 0.0f) ? s_dn : s;
  s = (t_up > 0.0f) ? s_up : s;
  return s;
}

// Correctly rounded n/d for n = 0 or 2^-47 <= |n| <= 2^40 and 2^-40 <= d <= 2^40: the IEEE
// division's expansion (reciprocal estimate, one Newton step, quotient, two exact-residual
// corrections) without the operand scaling that only extreme exponents need.
__device__ __forceinline__ float div_rn_safe(float n, float d) {
  float y = __builtin_amdgcn_rcpf(d);
  const float e = __builtin_fmaf(-d, y, 1.0f);
  y = __builtin_fmaf(e, y, y);
  float q = n * y;
  float r = __builtin_fmaf(-d, q, n);
  q = __builtin_fmaf(r, y, q);
  r = __builtin_fmaf(-d, q, n);
  return __builtin_fmaf(r, y, q);
}

// Correctly rounded 1/d for 2^-40 <= d <= 2^40: reciprocal estimate, one Newton step, two
// exact-residual corrections -- the IEEE division's expansion without the operand scaling that
// only extreme exponents need.
__device__ __forceinline__ float rcp_rn_safe(float d) {
  float y = __builtin_amdgcn_rcpf(d);
  const float e = __builtin_fmaf(-d, y, 1.0f);
  y = __builtin_fmaf(e, y, y);
  float r = __builtin_fmaf(-d, y, 1.0f);
  const float q = __builtin_fmaf(r, y, y);
  r = __builtin_fmaf(-d, q, 1.0f);
  return __builtin_fmaf(r, y, q);
}
// 2^-40 <= x <= 2^40, for x >= 0: positive floats order like their bit patterns
__device__ __forceinline__ bool in_safe_range(float x) { return f2u(x) - 0x2B800000u <= 0x53800000u - 0x2B800000u; }

// ------------------------------------------------------------------ update
struct UpdateArgs {
  float ibc1, ibc2, eps, lr, decay;
};

// theta' = theta*decay - lr * (mt / den), with the quotient computed either by the correctly
// rounded division, or (FAST) from the correctly rounded reciprocal rden = 1/den by two
// residual corrections, which gives the same correctly rounded quotient when no intermediate
// underflows or overflows (the caller checks the ranges that guarantee it).
template <bool FAST>
__device__ __forceinline__ float updated_param(float theta, float mt, float den, float rden, const UpdateArgs& u) {
  float ratio;
  if (FAST) {
    const float q0 = mt * rden;
    const float r0 = __builtin_fmaf(-den, q0, mt);
    const float q1 = __builtin_fmaf(r0, rden, q0);
    const float r1 = __builtin_fmaf(-den, q1, mt);
    ratio = __builtin_fmaf(r1, rden, q1);
  } else {
    ratio = mt / den;
  }
  const float upd = u.lr * ratio;
  const float dec = theta * u.decay;
  return dec - upd;
}

// Logarithmic quantization of v fused with the parameter update, for any width.  The code is the
// number of thresholds at or below rho = v/blockmax, found with one bucket lookup and one compare
// on the bit pattern of rho.  The update needs den = sqrt(vq*ibc2) + eps of the quantized value
// vq, which takes only 2^b values per block: with TABLE they (and their reciprocals) are read from
// the per-wave table DEN, indexed by (row, block, code); otherwise they are computed per element.
// mq holds the quantized first moments; theta is replaced by the new parameters.
template <int STATS, bool TAIL, bool TABLE, bool FAST>
__device__ __forceinline__ void quant2_update(const float (&v)[8], const float (&mq)[8], float (&theta)[8],
                                              uint32_t (&code)[8], const float (&sn)[2], const float (&inv)[2],
                                              const float* Lreg, uint32_t l_base, const uint2* VQ, const float2* DEN,
                                              const uint32_t (&den_row)[2], const UpdateArgs& u, uint32_t q, int lane,
                                              uint32_t n_valid, LaneStats<STATS>& st) {
  float sv_err = 0.0f;  // this quarter's part of the lane's sum of squared quantization errors
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const int i = n >> 2;
    const float rho = v[n] * inv[i];
    const uint32_t bits = f2u(rho);
    const uint32_t idx = __builtin_elementwise_sub_sat(bits >> kVqShift, kVqLow);  // rho <= 1: never past the last bucket
    const uint2 e = VQ[idx];
    uint32_t c = e.y + (bits >= e.x ? 1u : 0u);
    if (TAIL && !is_valid(n, q, lane, n_valid)) c = 0;
    code[n] = c;
    if (STATS == 1) {
      float vq = sn[i] * lds_at(Lreg, (c << 2) | l_base);
      if (TAIL && !is_valid(n, q, lane, n_valid)) vq = 0.0f;
      const float d = v[n] - vq;
      sv_err = __builtin_fmaf(d, d, sv_err);
    }
    const float mt = mq[n] * u.ibc1;
    if (TABLE) {
      const float2 dr = DEN[den_row[i] + c];
      theta[n] = updated_param<FAST>(theta[n], mt, dr.x, dr.y, u);
    } else {
      const float vq = sn[i] * lds_at(Lreg, (c << 2) | l_base);
      const float vt = vq * u.ibc2;
      if (FAST) {
        const float den = sqrt_rn_safe(vt) + u.eps;
        const float upd = u.lr * div_rn_safe(mt, den);
        const float dec = theta[n] * u.decay;
        theta[n] = dec - upd;
      } else {
        const float den = __builtin_sqrtf(vt) + u.eps;
        theta[n] = updated_param<false>(theta[n], mt, den, 0.0f, u);
      }
    }
  }
  if (STATS == 1) st.add(kLVErr, lane, sv_err);
}

// ------------------------------------------------------------------ one quarter tile
// Lane L = (value vL = L>>4, lane group qL = L&15) owns one (state, row) pair's block scale:
// state = vL>>1, row = 2q + (vL&1), block within the row = qL >> (lgK-4).  A block's owners are
// 4, 8 or 16 neighbouring lanes of one 16-lane row, so their maxima combine by DPP lane swaps.
// bfloat16 rounding (to nearest, ties to even) of a finite float, kept as a float
__device__ __forceinline__ float bf16_rne(float x) {
  uint32_t u = f2u(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u2f(u & 0xFFFF0000u);
}

// MODE 0: widths stay as they are; 1: the launch changes widths (other destination buffers);
// 2: as 1, and states may have the wide formats: 32 bits = the fp32 value, 16 bits = its bfloat16
// rounding, stored in the same tile format with 32- or 16-bit codes and without scales.
template <bool BF16, int STATS, bool TAIL, int MODE>
__device__ __forceinline__ void process_quarter(const TensorDesc& d, uint32_t tile, uint32_t q, uint32_t n_valid,
                                                const StepArgs& a, const uint32_t* lds, uint32_t* ws, int lane,
                                                uint32_t& carry_m, uint32_t& carry_v, LaneStats<STATS>& st) {
  // Everything derived from the lane index and the block size is cheap to recompute.  Hide the two
  // from loop-invariant code motion, which would otherwise keep dozens of such values live across
  // the whole tile loop and spill them.
  asm volatile("" : "+v"(lane));
  uint32_t lgK = a.lgK;
  asm volatile("" : "+s"(lgK));
  constexpr bool XW = MODE >= 1, WIDE = MODE == 2;
  const uint32_t bm = d.bm, bv = d.bv;              // widths of the stored codes
  // widths this step writes: the same, unless the launch changes widths (XW)
  const uint32_t bmo = XW ? d.bm_out : bm, bvo = XW ? d.bv_out : bv;
  const size_t e0 = static_cast<size_t>(tile) * kTile + 512u * q;
  STQ_GLOBAL float* P = as_global(d.param + e0);
  // the quarter's first bit: word (q*b)>>2 of the lane's b words, bit 8*((q*b)&3)
  const uint32_t s0m = 8u * ((q * bm) & 3u), s0v = 8u * ((q * bv) & 3u);
  STQ_GLOBAL uint32_t* CM = as_global(d.m_codes + static_cast<size_t>(tile) * 64u * bm) + ((q * bm) >> 2) * 64;
  STQ_GLOBAL uint32_t* CV = as_global(d.v_codes + static_cast<size_t>(tile) * 64u * bv) + ((q * bv) >> 2) * 64;
  // where the new codes go: the same buffers at the same widths, or other buffers at the new widths
  const uint32_t s0mo = 8u * ((q * bmo) & 3u), s0vo = 8u * ((q * bvo) & 3u);
  STQ_GLOBAL uint32_t* CMO = XW ? as_global(d.m_out + static_cast<size_t>(tile) * 64u * bmo) + ((q * bmo) >> 2) * 64 : CM;
  STQ_GLOBAL uint32_t* CVO = XW ? as_global(d.v_out + static_cast<size_t>(tile) * 64u * bvo) + ((q * bvo) >> 2) * 64 : CV;
  const size_t sbase = static_cast<size_t>(tile) << (11 - lgK);  // scales per tile = 2048/K
  // the lane index as a 6-bit unsigned offset: global addresses become uniform base + 32-bit offset
  const uint32_t ul = static_cast<uint32_t>(lane) & 63u;
  const int vL = lane >> 4, qL = lane & 15;
  const uint32_t sidx = ((2u * q + static_cast<uint32_t>(vL & 1)) << (8 - lgK)) + (static_cast<uint32_t>(qL) >> (lgK - 4));
  STQ_GLOBAL float* SC = as_global((vL >> 1) ? d.v_scales : d.m_scales);

  // ---- loads for the moment phase --------------------------------------------
  const float sc_old = SC[sbase + sidx];
  constexpr int kMaxWords = WIDE ? 8 : 3;  // a quarter of a wide state is 4 or 8 whole words
  uint32_t lwm[kMaxWords], lwv[kMaxWords];
  {
    const uint32_t nwm = (s0m + 8u * bm + 31u) >> 5, nwv = (s0v + 8u * bv + 31u) >> 5;  // 1..3 words (4, 8 wide)
#pragma unroll
    for (int k = 0; k < kMaxWords; ++k) lwm[k] = (static_cast<uint32_t>(k) < nwm) ? CM[k * 64u + ul] : 0u;
#pragma unroll
    for (int k = 0; k < kMaxWords; ++k) lwv[k] = (static_cast<uint32_t>(k) < nwv) ? CV[k * 64u + ul] : 0u;
  }
  float g[8];
  {
    STQ_GLOBAL const float* G32 = as_global(static_cast<const float*>(d.grad) + e0);
    STQ_GLOBAL const uint16_t* G16 = as_global(static_cast<const uint16_t*>(d.grad) + e0);
    if (!TAIL) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if (BF16) {
          const u32x2 r = __builtin_nontemporal_load(&reinterpret_cast<STQ_GLOBAL const u32x2*>(G16 + 256 * i)[ul]);
          g[4 * i + 0] = u2f(r.x << 16); g[4 * i + 1] = u2f(r.x & 0xFFFF0000u);
          g[4 * i + 2] = u2f(r.y << 16); g[4 * i + 3] = u2f(r.y & 0xFFFF0000u);
        } else {
          const f32x4 r = __builtin_nontemporal_load(&reinterpret_cast<STQ_GLOBAL const f32x4*>(G32 + 256 * i)[ul]);
          g[4 * i + 0] = r.x; g[4 * i + 1] = r.y; g[4 * i + 2] = r.z; g[4 * i + 3] = r.w;
        }
      }
    } else {
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        float x = 0.0f;
        if (is_valid(n, q, lane, n_valid)) {
          const uint32_t idx = 256u * (n >> 2) + 4u * ul + (n & 3);
          x = BF16 ? u2f(static_cast<uint32_t>(G16[idx]) << 16) : G32[idx];
        }
        g[n] = x;
      }
    }
  }

  // old scales to every lane that needs them: lane j reads the 4 values of its lane group
  float* wsf = reinterpret_cast<float*>(ws);
  float* XR = wsf;                // [4][XS]
  float* SO = wsf + 4 * XS;       // [64] old scales at [lane group * 4 + value]
  float* SN = SO + 64;            // [64] new scales
  float* SI = SN + 64;            // [64] reciprocals of the new scales
  SO[qL * 4 + vL] = sc_old;
  wave_lds_sync();
  float som[2], sov[2];
  {
    const float4 a0 = *reinterpret_cast<const float4*>(SO + (lane >> 2) * 4);
    som[0] = a0.x; som[1] = a0.y; sov[0] = a0.z; sov[1] = a0.w;
  }

  if (STATS) {
    double sg_sum = 0.0, sg_abs = 0.0, sg_sq = 0.0;  // fp64 from the first addition (pads are zeros)
    float sg_max = 0.0f;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const double gd = static_cast<double>(g[n]);
      sg_sum += gd;
      sg_abs += __builtin_fabs(gd);
      sg_sq = __builtin_fma(gd, gd, sg_sq);
      sg_max = fmaxf(sg_max, fabsf(g[n]));
    }
    st.add_grad(kLGSum, lane, sg_sum);
    st.add_grad(kLGAbs, lane, sg_abs);
    st.add_grad(kLGSq, lane, sg_sq);
    st.max_grad(lane, sg_max);
  }

  // ---- moments: m_t = beta1*m_{t-1} + (1-beta1)*g ; v_t = beta2*v_{t-1} + (1-beta2)*g^2 ----
  const float* Rreg = reinterpret_cast<const float*>(lds) + kTabROff;  // value tables, see stq_tables.h
  const float* Lreg = reinterpret_cast<const float*>(lds) + kTabLOff;
  float m[8], v[8];
  {
    uint32_t off[8];
    float old[8];  // the stored moments m_{t-1}, then v_{t-1}
    if (WIDE && bm >= 16) {
#pragma unroll
      for (int n = 0; n < 8; ++n)
        old[n] = bm == 32 ? u2f(lwm[n]) : u2f((n & 1) ? (lwm[n >> 1] & 0xFFFF0000u) : (lwm[n >> 1] << 16));
    } else {
      STQ_SWITCH_BITS(bm, (unpack_offsets<B>(lwm, s0m, off)));
#pragma unroll
      for (int n = 0; n < 8; ++n) old[n] = som[n >> 2] * lds_at(Rreg, off[n]);
    }
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const float x = a.beta1 * old[n], y = a.omb1 * g[n];
      m[n] = x + y;
    }
    if (WIDE && bv >= 16) {
#pragma unroll
      for (int n = 0; n < 8; ++n)
        old[n] = bv == 32 ? u2f(lwv[n]) : u2f((n & 1) ? (lwv[n >> 1] & 0xFFFF0000u) : (lwv[n >> 1] << 16));
    } else {
      STQ_SWITCH_BITS(bv, (unpack_offsets<B>(lwv, s0v, off)));
#pragma unroll
      for (int n = 0; n < 8; ++n) old[n] = sov[n >> 2] * lds_at(Lreg, off[n]);
    }
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const float gg = g[n] * g[n];
      const float x = a.beta2 * old[n], y = a.omb2 * gg;
      v[n] = x + y;
    }
  }
  if (TAIL) {
#pragma unroll
    for (int n = 0; n < 8; ++n)
      if (!is_valid(n, q, lane, n_valid)) { m[n] = 0.0f; v[n] = 0.0f; }
  }

  if (STATS == 1) {
    // the moments' sums and sums of squares, taken here where few other values are live (their quantization
    // errors follow in the quantizer loops)
    float sm_sum = 0.0f, sm_sq = 0.0f, sv_sum = 0.0f, sv_sq = 0.0f;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      sm_sum += m[n];
      sm_sq = __builtin_fmaf(m[n], m[n], sm_sq);
      sv_sum += v[n];
      sv_sq = __builtin_fmaf(v[n], v[n], sv_sq);
    }
    st.add(kLMSum, lane, sm_sum);
    st.add(kLMSq, lane, sm_sq);
    st.add(kLVSum, lane, sv_sum);
    st.add(kLVSq, lane, sv_sq);
  }

  // ---- parameters: issued here so that they arrive while the block maxima are reduced ----
  // Parameters and gradients are touched once per step: non-temporal accesses keep them from
  // displacing the code and scale lines in the caches (measured: both the load and the store of
  // the parameters must carry the hint; on the code and scale streams it loses).
  float theta[8];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (!TAIL) {
      const f32x4 t = __builtin_nontemporal_load(&reinterpret_cast<STQ_GLOBAL const f32x4*>(P + 256 * i)[ul]);
      theta[4 * i] = t.x; theta[4 * i + 1] = t.y; theta[4 * i + 2] = t.z; theta[4 * i + 3] = t.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        theta[4 * i + e] = is_valid(4 * i + e, q, lane, n_valid) ? P[256u * i + 4u * ul + e] : 0.0f;
    }
  }

  // ---- block maxima: lane partials -> LDS transpose -> one owner lane per (state,row,block)
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float pm = fmaxf(fmaxf(fabsf(m[4 * i]), fabsf(m[4 * i + 1])), fmaxf(fabsf(m[4 * i + 2]), fabsf(m[4 * i + 3])));
    const float pv = fmaxf(fmaxf(v[4 * i], v[4 * i + 1]), fmaxf(v[4 * i + 2], v[4 * i + 3]));
    XR[i * XS + lane] = pm;
    XR[(2 + i) * XS + lane] = pv;
  }
  wave_lds_sync();
  // the maxima are non-negative, so they order like their bit patterns: integer max, no NaN handling
  float r;
  {
    const uint4 t0 = *reinterpret_cast<const uint4*>(XR + vL * XS + qL * 4);
    uint32_t rb = max(max(t0.x, t0.y), max(t0.z, t0.w));
    rb = max(rb, dpp_u32<kDppXor1>(rb));
    rb = max(rb, dpp_u32<kDppXor2>(rb));
    if (lgK >= 7) rb = max(rb, dpp_u32<kDppHalfMirror>(rb));
    if (lgK == 8) rb = max(rb, dpp_u32<kDppMirror>(rb));
    r = u2f(rb);
  }
  if (STATS == 1) {
    st.max_moment(lane, r);
  }
  // a block whose maximum is below the smallest normal number is stored as all-zero
  const float sc_new = (r < FLT_MIN) ? 0.0f : r;
  float sc_inv;
  if (__all(static_cast<int>(sc_new == 0.0f) | static_cast<int>(in_safe_range(sc_new)))) {
    sc_inv = (sc_new > 0.0f) ? rcp_rn_safe(sc_new) : 0.0f;
  } else {
    sc_inv = (sc_new > 0.0f) ? 1.0f / sc_new : 0.0f;
  }
  SN[qL * 4 + vL] = sc_new;
  SI[qL * 4 + vL] = sc_inv;
  {
    // a wide state has no scales: its owners store nothing
    const bool has_scale = !WIDE || (vL < 2 ? bmo : bvo) < 16;
    if (has_scale && (static_cast<uint32_t>(qL) & ((1u << (lgK - 4)) - 1u)) == 0u) SC[sbase + sidx] = sc_new;
  }
  wave_lds_sync();

  // ---- table of den = sqrt(vq*ibc2) + eps and 1/den per (row, block, second-moment code) ----
  // Used when a level serves at least four elements: entries = (512/K) << bv_out <= 128.  The table
  // takes the place of XR, whose last readers have finished.
  const UpdateArgs ua = {a.ibc1, a.ibc2, a.eps, a.lr, a.decay};
  const bool wide_m = WIDE && bmo >= 16, wide_v = WIDE && bvo >= 16;
  const uint32_t n_entries = wide_v ? 0xFFFFFFFFu : (512u >> lgK) << bvo;
  const bool use_table = n_entries <= kDenEntries;
  const uint32_t l_base = wide_v ? 0u : 4u << bvo;
  float2* DEN = reinterpret_cast<float2*>(XR);
  // The short forms of the quotient (and, without a table, of the square root) need every operand
  // in a range where no intermediate underflows or overflows.  The owner lanes check their scales:
  // m~ = (s_m*R)*ibc1 is 0 or at least s_m*ibc1/127; v~ = (s_v*L)*ibc2 is 0 or at least
  // s_v*ibc2*2^-16, so its root lies in [2^-40, 2^39] when s_v*ibc2 lies in [2^-64, 2^78].
  int bad_bits;
  if (vL < 2) {
    bad_bits = (static_cast<int>(sc_new == 0.0f) | static_cast<int>(in_safe_range(sc_new * a.ibc1))) ^ 1;
  } else {
    const float x = sc_new * a.ibc2;
    bad_bits = (static_cast<int>(sc_new == 0.0f) | static_cast<int>(f2u(x) - 0x1F800000u <= 0x66800000u - 0x1F800000u)) ^ 1;
  }
  const bool eps_ok = a.eps >= 0x1p-40f && a.eps <= 1.0f;
  bool fast_div;
  if (use_table) {
    // the scales are in range: the short forms build the table as well (their results are the correctly
    // rounded ones); else the IEEE routines do, and the quotient later takes the IEEE division too
    const bool short_forms = eps_ok && !__any(bad_bits);
    if (!short_forms) bad_bits = 1;
    for (uint32_t e = lane; e < n_entries; e += 64) {
      const uint32_t c = e & ((1u << bvo) - 1u), rg = e >> bvo;
      const uint32_t row = rg >> (8 - lgK), blk = rg & ((1u << (8 - lgK)) - 1u);
      const float sv = SN[((blk << (lgK - 4)) << 2) + 2 + row];
      const float vq = sv * lds_at(Lreg, (c << 2) | l_base);
      const float vt = vq * a.ibc2;
      float den, rden;
      if (short_forms) {
        den = sqrt_rn_safe(vt) + a.eps;  // vt is 0 or in [2^-80, 2^78]; den in [eps, 2^39 + 1]
        rden = rcp_rn_safe(den);
      } else {
        den = __builtin_sqrtf(vt) + a.eps;
        rden = 1.0f / den;
      }
      // the quotient's short form needs the correctly rounded reciprocal, which a divisor with an all-ones
      // mantissa may not have
      bad_bits |= static_cast<int>((f2u(den) & 0x7FFFFFu) == 0x7FFFFFu);
      DEN[e] = make_float2(den, rden);
    }
    fast_div = !__any(bad_bits);
    wave_lds_sync();
  } else {
    fast_div = eps_ok && !__any(bad_bits);
  }
  if (wide_m) fast_div = false;  // a wide first moment is not a multiple of a block scale: no range guarantee

  // ---- linear symmetric quantization of m; m is replaced by its quantized value ----
  if (wide_m) {
    float sm_err = 0.0f;
    uint32_t kept[8];
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const float mq = bmo == 32 ? m[n] : bf16_rne(m[n]);  // pads are 0 and stay 0
      if (STATS == 1) {
        const float dd = m[n] - mq;
        sm_err = __builtin_fmaf(dd, dd, sm_err);
      }
      m[n] = mq;
      kept[n] = f2u(mq);
    }
    if (STATS == 1) st.add(kLMErr, lane, sm_err);
    if (bmo == 32) {
#pragma unroll
      for (int n = 0; n < 8; ++n) CMO[n * 64u + ul] = kept[n];
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) CMO[k * 64u + ul] = (kept[2 * k] >> 16) | (kept[2 * k + 1] & 0xFFFF0000u);
    }
  } else {
    float sn[2], inv[2];
    {
      const float4 a0 = *reinterpret_cast<const float4*>(SN + (lane >> 2) * 4);
      const float4 b0 = *reinterpret_cast<const float4*>(SI + (lane >> 2) * 4);
      sn[0] = a0.x; sn[1] = a0.y; inv[0] = b0.x; inv[1] = b0.y;
    }
    const int qmax = (1 << (bmo - 1)) - 1;
    const float qmaxf = static_cast<float>(qmax);
    const uint32_t r_base = 4u << bmo;
    uint32_t code[8];
    float sm_err = 0.0f;  // this quarter's part of the lane's sum of squared quantization errors
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int i = n >> 2;
      const float t = (m[n] * inv[i]) * qmaxf;
      // round half to even: adding 1.5*2^23 leaves the integer in the low mantissa bits (|t| <= 127.5)
      const float rr = t + 12582912.0f;
      // |m| <= s and 1/s is within half an ulp, so |t| <= qmax*(1 + 2^-22) rounds to at most qmax:
      // the clamp of the quantizer's definition can never act and is left out
      uint32_t u = f2u(rr) - static_cast<uint32_t>(0x4B400000 - qmax);
      if (TAIL && !is_valid(n, q, lane, n_valid)) u = 0;
      code[n] = u;
      float mq = sn[i] * lds_at(Rreg, (u << 2) | r_base);
      if (STATS == 1) {
        if (TAIL && !is_valid(n, q, lane, n_valid)) mq = 0.0f;
        const float dd = m[n] - mq;
        sm_err = __builtin_fmaf(dd, dd, sm_err);
      }
      m[n] = mq;
    }
    if (STATS == 1) st.add(kLMErr, lane, sm_err);
    STQ_SWITCH_BITS(bmo, (pack_store<B>(code, CMO, s0mo, carry_m, ul)));
  }

  // ---- logarithmic quantization of v and the parameter update ----
  if (wide_v) {
    float sv_err = 0.0f;
    uint32_t kept[8];
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const float vq = bvo == 32 ? v[n] : bf16_rne(v[n]);
      if (STATS == 1) {
        const float dd = v[n] - vq;
        sv_err = __builtin_fmaf(dd, dd, sv_err);
      }
      kept[n] = f2u(vq);
      const float mt = m[n] * ua.ibc1;
      const float vt = vq * ua.ibc2;
      const float den = __builtin_sqrtf(vt) + ua.eps;
      theta[n] = updated_param<false>(theta[n], mt, den, 0.0f, ua);
    }
    if (STATS == 1) st.add(kLVErr, lane, sv_err);
    if (bvo == 32) {
#pragma unroll
      for (int n = 0; n < 8; ++n) CVO[n * 64u + ul] = kept[n];
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) CVO[k * 64u + ul] = (kept[2 * k] >> 16) | (kept[2 * k + 1] & 0xFFFF0000u);
    }
  } else {
    float sn[2], inv[2];
    {
      const float4 a1 = *reinterpret_cast<const float4*>(SN + (lane >> 2) * 4);
      const float4 b1 = *reinterpret_cast<const float4*>(SI + (lane >> 2) * 4);
      sn[0] = a1.z; sn[1] = a1.w; inv[0] = b1.z; inv[1] = b1.w;
    }
    const uint2* VQ = reinterpret_cast<const uint2*>(lds + kTabVqOff) + (bvo - 2) * kVqBuckets;
    // den table entry ((row*G + block) << bv_out) + c, G = 256/K blocks per row
    uint32_t den_row[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
      den_row[i] = (((static_cast<uint32_t>(i) << (8 - lgK)) + (static_cast<uint32_t>(lane) >> (lgK - 2))) << bvo);
    uint32_t code[8];
    if (use_table) {
      if (fast_div)
        quant2_update<STATS, TAIL, true, true>(v, m, theta, code, sn, inv, Lreg, l_base, VQ, DEN, den_row, ua, q, lane, n_valid, st);
      else
        quant2_update<STATS, TAIL, true, false>(v, m, theta, code, sn, inv, Lreg, l_base, VQ, DEN, den_row, ua, q, lane, n_valid, st);
    } else {
      if (fast_div)
        quant2_update<STATS, TAIL, false, true>(v, m, theta, code, sn, inv, Lreg, l_base, VQ, DEN, den_row, ua, q, lane, n_valid, st);
      else
        quant2_update<STATS, TAIL, false, false>(v, m, theta, code, sn, inv, Lreg, l_base, VQ, DEN, den_row, ua, q, lane, n_valid, st);
    }
    STQ_SWITCH_BITS(bvo, (pack_store<B>(code, CVO, s0vo, carry_v, ul)));
  }

#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (!TAIL) {
      __builtin_nontemporal_store(f32x4{theta[4 * i], theta[4 * i + 1], theta[4 * i + 2], theta[4 * i + 3]},
                                  &reinterpret_cast<STQ_GLOBAL f32x4*>(P + 256 * i)[ul]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (is_valid(4 * i + e, q, lane, n_valid)) P[256u * i + 4u * ul + e] = theta[4 * i + e];
    }
  }
}

// The descriptor table is never written while a step runs: reading it through the constant
// address space gives scalar loads, so everything derived from a descriptor (all base addresses)
// lives in scalar registers.
#define STQ_CONSTANT __attribute__((address_space(4)))
__device__ __forceinline__ TensorDesc load_desc(const TensorDesc* table, uint32_t l) {
  const STQ_CONSTANT uint64_t* p = (const STQ_CONSTANT uint64_t*)(table + l);
  static_assert(sizeof(TensorDesc) == 96, "descriptor layout");
  uint64_t w[sizeof(TensorDesc) / 8];
#pragma unroll
  for (size_t i = 0; i < sizeof(TensorDesc) / 8; ++i) w[i] = p[i];
  TensorDesc d;
  __builtin_memcpy(&d, w, sizeof(TensorDesc));
  return d;
}
__device__ __forceinline__ uint32_t desc_tile_begin(const TensorDesc* table, uint32_t l) {
  const STQ_CONSTANT uint32_t* p = (const STQ_CONSTANT uint32_t*)(&table[l].tile_begin);
  return *p;
}

// -------------------------------------------------------------- step kernel
// Order of the work.  A unit is a tile (or a quarter tile, see below).  Two schedules:
//  * tickets (a.sched set): the workgroups of the launch draw tickets from one counter in device memory.
//    Ticket k stands for the kWaves consecutive units k*kWaves .. k*kWaves + kWaves-1, one per wave; the
//    waves of a workgroup meet at a barrier before they go on to the next ticket (drawn while they work on
//    the current one, so its latency is hidden; a workgroup's first ticket is its own index).  The waves of a
//    workgroup then read and write neighbouring tiles at the same time, and the chip as a whole works inside
//    one compact window of the launch-wide order that moves forward in order.  On multi-gigabyte workloads the
//    memory system gives 10-15 % more bandwidth to this than to waves that each walk their own stripe of the
//    arrays at their own pace; on small ones the barrier costs more than the order gains.
//  * stripes (a.sched null): wave w of W takes the chunks w, w+W, w+2W, ... of `chunk` consecutive units.
//    The variants that collect statistics use it with few, long chunks (a wave flushes its sums to the
//    tensor's global slots whenever its next unit lies in another tensor), the plain one with chunk 1 or 4.
// The ticket counter resets itself: the last workgroup to leave the kernel clears it (and the count of
// workgroups that have left), so every launch -- also a replayed one -- finds both at zero.
// STATS 1 (all statistics) and 2 (the gradient's only) stay within the plain kernel's budget of 80 registers
// and a third of a CU's LDS: their running sums live in LDS and nothing derived from the lane index is kept
// across the tile loop (see LaneStats).  Only the wide-state variant (MODE 2) runs two workgroups per CU.
template <bool BF16, int STATS, int MODE>
__global__ __launch_bounds__(64 * kWavesPerGroup, MODE == 2 ? 4 : 6) void step_kernel(const StepArgs a) {
  constexpr int kWaves = kWavesPerGroup;
  __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsWords + kWavesPerGroup * LaneStats<STATS>::kWords];
  __shared__ uint32_t drawn[2];  // the ticket being worked on and the next one, alternating
  // statistics of the two tickets in flight, one record per wave
  __shared__ TicketRecord<STATS> ticket_rec[2][kWavesPerGroup];
  const bool tickets = a.sched != nullptr;
  if (threadIdx.x == 0) drawn[0] = blockIdx.x;
  // the value tables of every width (4 KB), the search table of the second-moment widths this launch can write
  for (int i = threadIdx.x; i < kTabVqOff; i += 64 * kWaves) lds[i] = a.tables[i];
  for (int b = kMinBits; b <= kMaxBits; ++b) {
    if (!((a.v_widths >> b) & 1u)) continue;
    const int base = kTabVqOff + (b - kMinBits) * kVqBuckets * 2;
    for (int i = threadIdx.x; i < kVqBuckets * 2; i += 64 * kWaves) lds[base + i] = a.tables[base + i];
  }
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t* ws = lds + kTabWords + wave * kWaveScratch;
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * kWaves;
  // A unit of scheduling is a tile; in a launch too small to occupy the waves with whole tiles, and
  // whose widths are all multiples of 4 bits (a quarter's codes then start and end on word
  // boundaries), it is a quarter tile.
  const uint32_t qs = a.quarter_units ? 2u : 0u;
  const uint64_t total_units = static_cast<uint64_t>(a.total_tiles) << qs;
  const uint64_t C = a.chunk;
  uint64_t stripe = (static_cast<uint64_t>(blockIdx.x) * kWaves + wave) * C;  // next chunk of this wave (stripes)
  const uint32_t n_tickets = static_cast<uint32_t>((total_units + kWaves - 1) / kWaves);
  uint32_t turn = 0;         // which of drawn[] is current (tickets)
  uint32_t next_ticket = 0;  // thread 0: the ticket drawn for the next round

  uint32_t l = 0;
  bool have_desc = false;
  TensorDesc d;
  LaneStats<STATS> st;
  st.acc = STATS ? reinterpret_cast<float*>(lds + kLdsWords + wave * LaneStats<STATS>::kWords) : nullptr;
  st.tiles = 0;
  if (STATS) st.clear_all(lane);
  for (;;) {
    uint64_t c_begin, c_end;
    if (tickets) {
      const uint32_t cur = __builtin_amdgcn_readfirstlane(drawn[turn]);
      if (cur >= n_tickets) break;  // the same for every wave of the workgroup
      // the counter hands out the tickets from gridDim.x on
      if (threadIdx.x == 0) next_ticket = gridDim.x + __hip_atomic_fetch_add(a.sched, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      c_begin = static_cast<uint64_t>(cur) * kWaves + wave;
      c_end = min(c_begin + 1, total_units);
    } else {
      if (stripe >= total_units) break;
      c_begin = stripe;
      c_end = min(stripe + C, total_units);
      stripe += n_waves * C;
    }
    for (uint64_t u = c_begin; u < c_end; ++u) {
      const uint32_t t = static_cast<uint32_t>(u >> qs);
      const uint32_t q_begin = qs ? static_cast<uint32_t>(u & 3u) : 0u, q_end = qs ? q_begin + 1u : 4u;
      if (!have_desc) {
        // tensor holding the wave's first tile: last l with tile_begin <= tile
        uint32_t lo = 0, hi = a.n_tensors - 1;
        while (lo < hi) {
          const uint32_t mid = (lo + hi + 1) >> 1;
          if (desc_tile_begin(a.desc, mid) <= t) lo = mid; else hi = mid - 1;
        }
        l = __builtin_amdgcn_readfirstlane(lo);
        d = load_desc(a.desc, l);
        have_desc = true;
      }
      if (t >= d.tile_begin + d.n_tiles) {  // t < total_tiles, so a later tensor holds it
        if (STATS && !tickets) flush_stats(st, a.stats + static_cast<size_t>(l) * kStatSlots, lane);
        do {
          ++l;
          d = load_desc(a.desc, l);
        } while (t >= d.tile_begin + d.n_tiles);
      }
      const uint32_t tile = t - d.tile_begin;
      const uint64_t left = d.numel - static_cast<uint64_t>(tile) * kTile;
      uint32_t carry_m = 0, carry_v = 0;
      if (left >= static_cast<uint64_t>(kTile)) {
#pragma nounroll
        for (uint32_t q = q_begin; q < q_end; ++q)
          process_quarter<BF16, STATS, false, MODE>(d, tile, q, kTile, a, lds, ws, lane, carry_m, carry_v, st);
      } else {
#pragma nounroll
        for (uint32_t q = q_begin; q < q_end; ++q)
          process_quarter<BF16, STATS, true, MODE>(d, tile, q, static_cast<uint32_t>(left), a, lds, ws, lane, carry_m,
                                                   carry_v, st);
      }
      if (STATS && tickets) {
        if constexpr (STATS != 0) {
          // does the ticket's first unit lie in this wave's tensor?  (it cannot lie behind it: units only grow)
          const uint32_t t_first = static_cast<uint32_t>((c_begin - wave) >> qs);
          ticket_stats_tile(st, &ticket_rec[turn][wave], t_first >= d.tile_begin, a.stats + static_cast<size_t>(l) * kStatSlots, lane);
        }
      } else if (STATS && ++st.tiles == kStatFlushTiles) {
        widen_stats(st, lane);
      }
    }
    if (tickets) {
      if constexpr (STATS != 0) {
        // a wave without a unit in this ticket (the launch's last one) leaves an empty record
        constexpr int kRecordDoubles = sizeof(TicketRecord<STATS>) / 8;
        if (c_begin >= c_end && lane < kRecordDoubles) reinterpret_cast<double*>(&ticket_rec[turn][wave])[lane] = 0.0;
      }
      if (threadIdx.x == 0) drawn[turn ^ 1u] = next_ticket;
      __syncthreads();  // the workgroup goes on together
      if constexpr (STATS != 0) {
        // wave 0 worked on the ticket's first unit: its l is that unit's tensor
        if (wave == 0) ticket_stats_flush(ticket_rec[turn], a.stats + static_cast<size_t>(l) * kStatSlots, lane);
      }
      turn ^= 1u;
    }
  }
  if (STATS && !tickets && have_desc) flush_stats(st, a.stats + static_cast<size_t>(l) * kStatSlots, lane);
  if (tickets && threadIdx.x == 0) {
    // every ticket this workgroup drew precedes its leaving; the last one to leave has seen all others leave
    const uint32_t left_before = __hip_atomic_fetch_add(a.sched + 1, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (left_before == gridDim.x - 1u) {
      __hip_atomic_store(a.sched, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.sched + 1, 0u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace

template <int MODE, int STATS>
static void launch_variant(const StepArgs& a, bool grad_bf16, dim3 grid, dim3 block, hipStream_t s) {
  if (grad_bf16) hipLaunchKernelGGL((step_kernel<true, STATS, MODE>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((step_kernel<false, STATS, MODE>), grid, block, 0, s, a);
}

template <int MODE>
static void launch_mode(const StepArgs& a, bool grad_bf16, int stats, dim3 grid, dim3 block, hipStream_t s) {
  if (stats == 1) launch_variant<MODE, 1>(a, grad_bf16, grid, block, s);
  else if (stats == 2) launch_variant<MODE, 2>(a, grad_bf16, grid, block, s);
  else launch_variant<MODE, 0>(a, grad_bf16, grid, block, s);
}

// mode: 0 in place at unchanged widths, 1 widths change, 2 as 1 with 16- or 32-bit states
// stats: 0 none, 1 every statistic, 2 the gradient's only
int launch_step(const StepArgs& a, bool grad_bf16, int stats, int mode, uint32_t groups, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(groups), block(64 * kWavesPerGroup);
  if (mode == 2) launch_mode<2>(a, grad_bf16, stats, grid, block, s);
  else if (mode == 1) launch_mode<1>(a, grad_bf16, stats, grid, block, s);
  else launch_mode<0>(a, grad_bf16, stats, grid, block, s);
  return static_cast<int>(hipGetLastError());
}

}  // namespace stq
