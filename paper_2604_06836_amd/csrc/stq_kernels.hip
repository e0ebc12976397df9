// Small gfx950 kernels around the quantized Adam step: the initial state m_0 = v_0 = 0 of
// Algorithm 1, the conversion of stored codes when a layer's bit-width changes, and a fill.
// The step kernel itself is in stq_step.hip.
#include <hip/hip_runtime.h>

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
  const uint32_t qmax = (1u << (a.bm - 1)) - 1u;
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
// Width change of one state: every code goes through a 256-entry table; pad codes stay 0.
// One thread per (tile, lane) streams its b_old words into b_new words.
__global__ __launch_bounds__(256) void repack_kernel(const RepackArgs a) {
  __shared__ uint32_t lut[256];
  lut[threadIdx.x] = a.lut[threadIdx.x];
  __syncthreads();
  const uint64_t gid = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  const uint64_t tile = gid >> 6;
  const uint32_t lane = gid & 63;
  if (tile >= a.n_tiles) return;
  const uint32_t* src = a.src + tile * 64 * a.b_old + lane;
  uint32_t* dst = a.dst + tile * 64 * a.b_new + lane;
  const uint32_t mask = (1u << a.b_old) - 1u;
  uint64_t in = 0, out = 0;
  uint32_t in_bits = 0, out_bits = 0, ip = 0, op = 0;
  for (uint32_t n = 0; n < 32; ++n) {
    if (in_bits < a.b_old) {
      in |= static_cast<uint64_t>(src[64 * ip++]) << in_bits;
      in_bits += 32;
    }
    const uint32_t code = static_cast<uint32_t>(in) & mask;
    in >>= a.b_old;
    in_bits -= a.b_old;
    const uint64_t idx = tile * kTile + 256 * (n >> 2) + 4 * lane + (n & 3);
    const uint32_t c2 = idx < a.numel ? lut[code] : 0u;
    out |= static_cast<uint64_t>(c2) << out_bits;
    out_bits += a.b_new;
    if (out_bits >= 32) {
      dst[64 * op++] = static_cast<uint32_t>(out);
      out >>= 32;
      out_bits -= 32;
    }
  }
}

// Many width changes in one launch.  Wave w of W takes tiles w, w+W, ... of the launch-wide tile
// order; when it enters another job it reloads that job's conversion table into its LDS slice.
__global__ __launch_bounds__(256) void repack_many_kernel(const RepackManyArgs a) {
  __shared__ uint32_t lut_all[4][256];
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t* lut = lut_all[wave];
  const uint32_t n_waves = gridDim.x * 4;
  uint32_t t = blockIdx.x * 4 + wave;
  if (t >= a.total_tiles) return;
  // job holding tile t: last j with tile_begin <= t
  uint32_t lo = 0, hi = a.n_jobs - 1;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) >> 1;
    if (a.jobs[mid].tile_begin <= t) lo = mid; else hi = mid - 1;
  }
  uint32_t j = lo, loaded = 0xFFFFFFFFu;
  for (; t < a.total_tiles; t += n_waves) {
    while (t >= a.jobs[j].tile_begin + a.jobs[j].n_tiles) ++j;  // t < total_tiles: a later job holds it
    const RepackJob job = a.jobs[j];
    if (loaded != job.lut) {
      __builtin_amdgcn_wave_barrier();  // the previous tile's table reads are done (same wave, in order)
      for (uint32_t k = lane; k < 256; k += 64) lut[k] = a.luts[job.lut * 256 + k];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      loaded = job.lut;
    }
    const uint64_t tile = t - job.tile_begin;
    const uint32_t* src = job.src + tile * 64 * job.b_old + lane;
    uint32_t* dst = job.dst + tile * 64 * job.b_new + lane;
    const uint32_t mask = (1u << job.b_old) - 1u;
    uint64_t in = 0, out = 0;
    uint32_t in_bits = 0, out_bits = 0, ip = 0, op = 0;
    for (uint32_t n = 0; n < 32; ++n) {
      if (in_bits < job.b_old) {
        in |= static_cast<uint64_t>(src[64 * ip++]) << in_bits;
        in_bits += 32;
      }
      const uint32_t code = static_cast<uint32_t>(in) & mask;
      in >>= job.b_old;
      in_bits -= job.b_old;
      const uint64_t idx = tile * kTile + 256 * (n >> 2) + 4 * lane + (n & 3);
      const uint32_t c2 = idx < job.numel ? lut[code] : 0u;
      out |= static_cast<uint64_t>(c2) << out_bits;
      out_bits += job.b_new;
      if (out_bits >= 32) {
        dst[64 * op++] = static_cast<uint32_t>(out);
        out >>= 32;
        out_bits -= 32;
      }
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, uint64_t words) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < words) p[i] = 0u;
}

}  // namespace

// -------------------------------------------------------------------- launchers
int launch_zero(const ZeroArgs& a, void* stream) {
  const uint64_t threads = static_cast<uint64_t>(a.n_tiles) * 64;
  hipLaunchKernelGGL(zero_kernel, dim3(static_cast<uint32_t>((threads + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), a);
  return static_cast<int>(hipGetLastError());
}

int launch_repack(const RepackArgs& a, void* stream) {
  const uint64_t threads = static_cast<uint64_t>(a.n_tiles) * 64;
  hipLaunchKernelGGL(repack_kernel, dim3(static_cast<uint32_t>((threads + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), a);
  return static_cast<int>(hipGetLastError());
}

int launch_repack_many(const RepackManyArgs& a, uint32_t groups, void* stream) {
  hipLaunchKernelGGL(repack_many_kernel, dim3(groups), dim3(256), 0, static_cast<hipStream_t>(stream), a);
  return static_cast<int>(hipGetLastError());
}

int launch_fill_zero(uint32_t* p, uint64_t words, void* stream) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<uint32_t>((words + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), p, words);
  return static_cast<int>(hipGetLastError());
}

}  // namespace stq
