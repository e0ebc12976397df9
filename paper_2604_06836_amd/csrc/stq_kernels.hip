// Small gfx950 kernels around the quantized Adam step: the initial state m_0 = v_0 = 0 of
// Algorithm 1, the conversion of stored codes when a layer's bit-width changes, the statistics of the
// gradients alone, and a fill.
// The step kernel itself is in stq_step.hip.
#include <hip/hip_runtime.h>

#include <utility>

#include <cstdint>

#include "stq_device.h"
#include "stq_tables.h"

#pragma clang fp contract(off)

namespace stq {
namespace {

// ------------------------------------------------------- initial state kernel
// m_0 = v_0 = 0: first-moment codes hold the zero code qmax (pad elements 0), second-moment
// codes and all scales are 0.  One thread per (tile, lane).
__global__ __launch_bounds__(256) void zero_kernel(const ZeroArgs a) {
  const uint64_t gid = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  const uint64_t tile = gid >> 6;
  const uint32_t lane = gid & 63;
  if (tile >= a.n_tiles) return;
  const uint32_t qmax = a.bm >= 16 ? 0u : (1u << (a.bm - 1)) - 1u;  // a 16- or 32-bit state stores +0.0
  for (uint32_t p = 0; p < a.bm; ++p) {
    uint32_t word = 0;
    for (uint32_t n = 0; n < 32; ++n) {
      const uint64_t idx = tile * kTile + 256 * (n >> 2) + 4 * lane + (n & 3);
      const uint32_t code = idx < a.numel ? qmax : 0u;
      const uint32_t bit = n * a.bm;               // stream position of the code
      const int rel = static_cast<int>(bit) - static_cast<int>(32 * p);
      if (rel >= 32 || rel + static_cast<int>(a.bm) <= 0) continue;
      word |= rel >= 0 ? (code << rel) : (code >> (-rel));
    }
    a.m_codes[tile * 64 * a.bm + p * 64 + lane] = word;
  }
  for (uint32_t p = 0; p < a.bv; ++p) a.v_codes[tile * 64 * a.bv + p * 64 + lane] = 0u;
  if (lane < a.scales_per_tile) {
    a.m_scales[tile * a.scales_per_tile + lane] = 0.0f;
    a.v_scales[tile * a.scales_per_tile + lane] = 0.0f;
  }
}

// --------------------------------------------------------------- re-pack kernel
// Width change of stored states: every code goes through a 256-entry table; pad codes stay 0.
// The lane's 32 codes of width B out of / into its B stream words; all shifts are compile-time.
// Pointers that arrive through the job table are loaded from memory, so the compiler cannot see that they
// are global; say so, to get global_load/global_store instead of flat accesses.
#define STQ_GLOBAL __attribute__((address_space(1)))
// Bits [SH, SH+B) of x in one instruction (from the plain expression the compiler makes a shift and a mask).
template <int SH, int B>
__device__ __forceinline__ uint32_t bit_field(uint32_t x) {
  uint32_t r;
  asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "n"(SH), "n"(B));
  return r;
}
// code N of a lane's stream words
template <int B, int N>
__device__ __forceinline__ uint32_t extract(const uint32_t (&w)[B]) {
  constexpr int off = N * B, p = off >> 5, sh = off & 31;
  if constexpr (sh + B <= 32) {
    return bit_field<sh, B>(w[p]);
  } else {  // a code that straddles two words: align it first
    return bit_field<0, B>(__builtin_amdgcn_alignbit(w[p + 1], w[p], static_cast<uint32_t>(sh)));
  }
}
template <int B, int... N>
__device__ __forceinline__ void extract_all(const uint32_t (&w)[B], uint32_t (&code)[32], std::integer_sequence<int, N...>) {
  ((code[N] = extract<B, N>(w)), ...);
}
template <int B>
__device__ __forceinline__ void unpack32(const STQ_GLOBAL uint32_t* src, uint32_t (&code)[32]) {
  uint32_t w[B];
#pragma unroll
  for (int p = 0; p < B; ++p) w[p] = src[64 * p];
  extract_all<B>(w, code, std::make_integer_sequence<int, 32>{});
}

template <int B>
__device__ __forceinline__ void pack32(const uint32_t (&code)[32], STQ_GLOBAL uint32_t* dst) {
  uint32_t w[B];
#pragma unroll
  for (int p = 0; p < B; ++p) w[p] = 0u;
#pragma unroll
  for (int n = 0; n < 32; ++n) {
    const int off = n * B, p = off >> 5, sh = off & 31;
    if (sh == 0) w[p] = code[n]; else w[p] |= code[n] << sh;
    if (sh + B > 32) w[p + 1] = code[n] >> (32 - sh);  // first bits of the next word
  }
#pragma unroll
  for (int p = 0; p < B; ++p) dst[64 * p] = w[p];
}

#define STQ_SWITCH_WIDTH(bits, CALL)       \
  switch (bits) {                          \
    case 2: { constexpr int B = 2; CALL; } break; \
    case 3: { constexpr int B = 3; CALL; } break; \
    case 4: { constexpr int B = 4; CALL; } break; \
    case 5: { constexpr int B = 5; CALL; } break; \
    case 6: { constexpr int B = 6; CALL; } break; \
    case 7: { constexpr int B = 7; CALL; } break; \
    default: { constexpr int B = 8; CALL; } break; \
  }

// The job table is not written while the kernel runs: reading it through the constant address
// space gives scalar loads.
#define STQ_CONSTANT __attribute__((address_space(4)))
__device__ __forceinline__ RepackJob load_job(const RepackJob* table, uint32_t j) {
  const STQ_CONSTANT uint64_t* p = (const STQ_CONSTANT uint64_t*)(table + j);
  static_assert(sizeof(RepackJob) == 48, "job layout");
  uint64_t w[6];
#pragma unroll
  for (int i = 0; i < 6; ++i) w[i] = p[i];
  RepackJob r;
  __builtin_memcpy(&r, w, sizeof(RepackJob));
  return r;
}
__device__ __forceinline__ uint32_t job_tile_begin(const RepackJob* table, uint32_t j) {
  return *(const STQ_CONSTANT uint32_t*)(&table[j].tile_begin);
}

// Many width changes in one launch.  One wave per workgroup; wave w of W takes the chunks w, w+W, ... of
// kRepackChunk consecutive tiles of the launch-wide tile order; when it enters a job with another conversion
// table it reloads its table.  The table sits at LDS address 0 as 256 bytes (new codes have at most 8 bits), so
// an old code is the address of its new code as it comes out of the bit-field extraction: one vector
// instruction per code to unpack, none to look up, one to pack -- the kernel moves (b_old + b_new)/8 bytes per
// element and was bound by instruction issue with a word table behind a per-wave base address.
__global__ __launch_bounds__(64) void repack_many_kernel(const RepackManyArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[256];  // the kernel's only LDS variable: address 0
  const uint32_t lane = threadIdx.x;
  const uint64_t n_waves = gridDim.x;
  uint64_t base = static_cast<uint64_t>(blockIdx.x) * kRepackChunk;
  if (base >= a.total_tiles) return;
  // job holding the first tile: last j with tile_begin <= base
  uint32_t lo = 0, hi = a.n_jobs - 1;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) >> 1;
    if (job_tile_begin(a.jobs, mid) <= static_cast<uint32_t>(base)) lo = mid; else hi = mid - 1;
  }
  uint32_t j = lo, loaded = 0xFFFFFFFFu;
  RepackJob job = load_job(a.jobs, j);
  for (; base < a.total_tiles; base += n_waves * kRepackChunk) {
   const uint32_t c_end = static_cast<uint32_t>(min(base + kRepackChunk, static_cast<uint64_t>(a.total_tiles)));
   for (uint32_t t = static_cast<uint32_t>(base); t < c_end; ++t) {
    while (t >= job.tile_begin + job.n_tiles) job = load_job(a.jobs, ++j);  // t < total_tiles: a later job holds it
    const uint32_t b_old = job.b_old, b_new = job.b_new, which = job.lut;
    if (loaded != which) {
      __builtin_amdgcn_wave_barrier();  // the previous tile's table reads are done (same wave, in order)
      // lane k packs entries 4k .. 4k+3 of the word table in device memory into one LDS word
      const uint4 e = *reinterpret_cast<const uint4*>(a.luts + which * 256 + 4 * lane);
      reinterpret_cast<uint32_t*>(lut)[lane] = e.x | (e.y << 8) | (e.z << 16) | (e.w << 24);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      loaded = which;
    }
    const uint64_t tile = t - job.tile_begin;
    const STQ_GLOBAL uint32_t* src = (const STQ_GLOBAL uint32_t*)(job.src + tile * 64 * b_old + lane);
    STQ_GLOBAL uint32_t* dst = (STQ_GLOBAL uint32_t*)(job.dst + tile * 64 * b_new + lane);
    uint32_t code[32];
    STQ_SWITCH_WIDTH(b_old, (unpack32<B>(src, code)));
#pragma unroll
    for (int n = 0; n < 32; ++n) code[n] = lut[code[n]];
    const uint64_t left = job.numel - tile * kTile;
    if (left < static_cast<uint64_t>(kTile)) {  // ragged last tile: pad codes are 0
      const uint32_t n_valid = static_cast<uint32_t>(left);
      // (the element offsets are computed here, where they are needed: derived from the plain lane index
      // they would be hoisted out of the loops and occupy two dozen registers throughout)
      uint32_t first = 4u * lane;
      asm volatile("" : "+v"(first));
#pragma unroll
      for (int n = 0; n < 32; ++n)
        if (256u * (n >> 2) + first + (n & 3) >= n_valid) code[n] = 0u;
    }
    STQ_SWITCH_WIDTH(b_new, (pack32<B>(code, dst)));
   }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, uint64_t words) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < words) p[i] = 0u;
}

// --------------------------------------------------- gradient statistics kernel
// The per-layer sums the bit-width decision reads (Eq. 2, 3, 8: sum g, sum |g|, sum g^2) and max |g|,
// from the gradients alone: for the order in which Algorithm 1 is written, where the decision of step t
// precedes that step's layer loop.  Streams the gradients once (HBM-bound).  Each wave takes one
// contiguous range of the launch-wide tile order; a lane keeps fp64 totals of its elements, and a wave adds
// its totals to the layer's accumulators once per layer it touched.
__device__ __forceinline__ void flush_grad_stats(double* slot, double s0, double s1, double s2, float mx, int lane) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    s0 += __shfl_xor(s0, o, 64);
    s1 += __shfl_xor(s1, o, 64);
    s2 += __shfl_xor(s2, o, 64);
    mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  }
  if (lane == 0) {
    atomicAdd(&slot[kGSum], s0);
    atomicAdd(&slot[kGAbsSum], s1);
    atomicAdd(&slot[kGSqSum], s2);
    // non-negative floats order like their bit patterns
    atomicMax(reinterpret_cast<uint32_t*>(&slot[kMaxGM]), __builtin_bit_cast(uint32_t, mx));
  }
}

typedef uint32_t gs_u32x2 __attribute__((ext_vector_type(2)));
typedef float gs_f32x4 __attribute__((ext_vector_type(4)));

template <bool BF16>
__global__ __launch_bounds__(256) void grad_stats_kernel(const TensorDesc* desc, uint32_t n_tensors,
                                                         uint32_t total_tiles, double* stats) {
  const int lane = threadIdx.x & 63;
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * 4;
  const uint64_t gw = static_cast<uint64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const uint64_t per_wave = (total_tiles + n_waves - 1) / n_waves;
  const uint64_t begin = gw * per_wave;
  const uint64_t end = begin + per_wave < total_tiles ? begin + per_wave : total_tiles;
  if (begin >= end) return;
  uint32_t lo = 0, hi = n_tensors - 1;  // last l with tile_begin <= begin
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) >> 1;
    if (desc[mid].tile_begin <= static_cast<uint32_t>(begin)) lo = mid; else hi = mid - 1;
  }
  uint32_t l = lo;
  uint32_t t_begin = desc[l].tile_begin, t_count = desc[l].n_tiles;
  uint64_t numel = desc[l].numel;
  const void* grad = desc[l].grad;
  double s0 = 0.0, s1 = 0.0, s2 = 0.0;
  float mx = 0.0f;
  for (uint64_t t = begin; t < end; ++t) {
    if (t >= static_cast<uint64_t>(t_begin) + t_count) {  // t < total_tiles, so a later tensor holds it
      flush_grad_stats(stats + static_cast<size_t>(l) * kStatSlots, s0, s1, s2, mx, lane);
      s0 = s1 = s2 = 0.0; mx = 0.0f;
      do {
        ++l;
        t_begin = desc[l].tile_begin; t_count = desc[l].n_tiles;
      } while (t >= static_cast<uint64_t>(t_begin) + t_count);
      numel = desc[l].numel;
      grad = desc[l].grad;
    }
    const uint64_t base = (t - t_begin) * kTile;
    const uint64_t left = numel - base;  // >= 1
    float g[32];
    if (left >= static_cast<uint64_t>(kTile)) {  // a whole tile: eight unconditional loads in flight
      if (BF16) {
        gs_u32x2 w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          w[i] = __builtin_nontemporal_load(reinterpret_cast<const gs_u32x2*>(static_cast<const uint16_t*>(grad) + base + 256u * i + 4u * lane));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          g[4 * i] = __builtin_bit_cast(float, w[i].x << 16); g[4 * i + 1] = __builtin_bit_cast(float, w[i].x & 0xFFFF0000u);
          g[4 * i + 2] = __builtin_bit_cast(float, w[i].y << 16); g[4 * i + 3] = __builtin_bit_cast(float, w[i].y & 0xFFFF0000u);
        }
      } else {
        gs_f32x4 w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          w[i] = __builtin_nontemporal_load(reinterpret_cast<const gs_f32x4*>(static_cast<const float*>(grad) + base + 256u * i + 4u * lane));
#pragma unroll
        for (int i = 0; i < 8; ++i) { g[4 * i] = w[i].x; g[4 * i + 1] = w[i].y; g[4 * i + 2] = w[i].z; g[4 * i + 3] = w[i].w; }
      }
    } else {  // the ragged last tile of a tensor: element by element
#pragma unroll
      for (int k = 0; k < 32; ++k) {
        const uint32_t off = 256u * (k >> 2) + 4u * lane + (k & 3);
        g[k] = 0.0f;
        if (off < left)
          g[k] = BF16 ? __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t*>(grad)[base + off]) << 16)
                      : static_cast<const float*>(grad)[base + off];
      }
    }
    // fp64 from the first addition: the decision compares scores with thresholds, and the variance of Eq. 3
    // is a difference of two of these sums (the kernel is bound by its one read of the gradients either way)
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      const double gd = static_cast<double>(g[k]);
      s0 += gd;
      s1 += __builtin_fabs(gd);
      s2 = __builtin_fma(gd, gd, s2);
      mx = fmaxf(mx, fabsf(g[k]));
    }
  }
  flush_grad_stats(stats + static_cast<size_t>(l) * kStatSlots, s0, s1, s2, mx, lane);
}

}  // namespace

// -------------------------------------------------------------------- launchers
int launch_zero(const ZeroArgs& a, void* stream) {
  const uint64_t threads = static_cast<uint64_t>(a.n_tiles) * 64;
  hipLaunchKernelGGL(zero_kernel, dim3(static_cast<uint32_t>((threads + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), a);
  return static_cast<int>(hipGetLastError());
}

int launch_repack_many(const RepackManyArgs& a, uint32_t groups, void* stream) {
  hipLaunchKernelGGL(repack_many_kernel, dim3(groups), dim3(64), 0, static_cast<hipStream_t>(stream), a);
  return static_cast<int>(hipGetLastError());
}

int launch_grad_stats(const TensorDesc* desc, uint32_t n_tensors, uint32_t total_tiles, double* stats, bool grad_bf16,
                      uint32_t groups, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (grad_bf16) hipLaunchKernelGGL(grad_stats_kernel<true>, dim3(groups), dim3(256), 0, s, desc, n_tensors, total_tiles, stats);
  else hipLaunchKernelGGL(grad_stats_kernel<false>, dim3(groups), dim3(256), 0, s, desc, n_tensors, total_tiles, stats);
  return static_cast<int>(hipGetLastError());
}

int launch_fill_zero(uint32_t* p, uint64_t words, void* stream) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<uint32_t>((words + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), p, words);
  return static_cast<int>(hipGetLastError());
}

}  // namespace stq
