// gfx950 kernels of the quantized Adam step (Algorithm 1 of the paper, per-layer loop body,
// with the block quantizers of Section 3.5), the initial state, and the width conversion.
//
// Arithmetic contract: IEEE binary32, every operation rounded on its own.  Build with
// -ffp-contract=off; division and square root are the correctly rounded ones.
//
// Work decomposition of the step: one wavefront owns one 2048-element tile at a time.  Lane j
// holds the 32 elements {256*i + 4*j + e}: every parameter / gradient access is a coalesced
// 16-byte (8-byte for bf16) per-lane row, the lane's 32 codes of a state are exactly b 32-bit
// words, and word p of all lanes is one contiguous 256-byte row of the code buffer.  A block of
// K = 64/128/256 consecutive elements is 16/32/64 neighbouring lanes of one row i.
#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "stq_device.h"
#include "stq_tables.h"

#pragma clang fp contract(off)

namespace stq {
namespace {

constexpr int XS = 68;                                // row stride (words) of the transpose scratch
constexpr int kWaveScratch = 16 * XS + 3 * 64;        // X[16][XS], old scales, new scales, reciprocals
constexpr int kLdsWords = kTabWords + kWavesPerGroup * kWaveScratch;

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// ---------------------------------------------------------------- bit streams
// Code n of width B sits at stream bits [n*B, n*B+B) of the lane's B words.
template <int B>
__device__ __forceinline__ uint32_t extract(const uint32_t (&w)[8], int n) {
  const int off = n * B, p = off >> 5, sh = off & 31;
  constexpr uint32_t mask = (1u << B) - 1u;
  if (sh + B <= 32) return (w[p] >> sh) & mask;
  return ((w[p] >> sh) | (w[p + 1] << (32 - sh))) & mask;
}

template <int B>
__device__ __forceinline__ void insert(uint32_t (&w)[8], int n, uint32_t code) {
  const int off = n * B, p = off >> 5, sh = off & 31;
  if (sh == 0) w[p] = code; else w[p] |= code << sh;
  if (sh + B > 32) w[p + 1] = code >> (32 - sh);  // first bits of the next word
}

// element n of lane `lane` is real (not pad) in a tile with n_valid elements
__device__ __forceinline__ bool is_valid(int n, int lane, uint32_t n_valid) {
  return static_cast<uint32_t>(256 * (n >> 2) + 4 * lane + (n & 3)) < n_valid;
}

// ------------------------------------------------------------- per-wave stats
struct LaneStats {
  double g_sum, g_abs, g_sq, m_sum, m_sq, m_err, v_sum, v_sq, v_err;
  float g_max, m_max, v_max;
  __device__ __forceinline__ void clear() {
    g_sum = g_abs = g_sq = m_sum = m_sq = m_err = v_sum = v_sq = v_err = 0.0;
    g_max = m_max = v_max = 0.0f;
  }
};

struct TileStats {  // fp32 partial sums of one lane over one tile (32 elements)
  float g_sum = 0, g_abs = 0, g_sq = 0, m_sum = 0, m_sq = 0, m_err = 0, v_sum = 0, v_sq = 0, v_err = 0;
  float g_max = 0, m_max = 0, v_max = 0;
};

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

__device__ void flush_stats(const LaneStats& s, double* slot, int lane) {
  const double t[9] = {wave_sum(s.g_sum), wave_sum(s.g_abs), wave_sum(s.g_sq),
                       wave_sum(s.m_sum), wave_sum(s.m_sq),  wave_sum(s.m_err),
                       wave_sum(s.v_sum), wave_sum(s.v_sq),  wave_sum(s.v_err)};
  const float gm = wave_max(s.g_max), mm = wave_max(s.m_max), vm = wave_max(s.v_max);
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < 9; ++k) atomicAdd(&slot[k], t[k]);
    // non-negative floats order like their bit patterns
    uint32_t* mx = reinterpret_cast<uint32_t*>(&slot[kMaxGM]);
    atomicMax(&mx[0], f2u(gm));
    atomicMax(&mx[1], f2u(mm));
    atomicMax(&mx[2], f2u(vm));
  }
}

// ------------------------------------------------------------------ tile arms
// Decode the stored first moment and form m_t = beta1*m_{t-1} + (1-beta1)*g.
template <int B>
__device__ __forceinline__ void moment1(const uint32_t (&w)[8], const float* R, const float (&so)[8],
                                        float beta1, float omb1, const float (&g)[32], float (&m)[32]) {
#pragma unroll
  for (int n = 0; n < 32; ++n) {
    const float mh = so[n >> 2] * R[extract<B>(w, n)];
    const float a = beta1 * mh, c = omb1 * g[n];
    m[n] = a + c;
  }
}

// Decode the stored second moment and form v_t = beta2*v_{t-1} + (1-beta2)*g^2.
template <int B>
__device__ __forceinline__ void moment2(const uint32_t (&w)[8], const float* L, const float (&so)[8],
                                        float beta2, float omb2, const float (&g)[32], float (&v)[32]) {
#pragma unroll
  for (int n = 0; n < 32; ++n) {
    const float vh = so[n >> 2] * L[extract<B>(w, n)];
    const float gg = g[n] * g[n];
    const float a = beta2 * vh, c = omb2 * gg;
    v[n] = a + c;
  }
}

// Linear symmetric quantization of m against the new block scales; m is replaced by its
// quantized value (the one the parameter update uses).
template <int B, bool STATS, bool TAIL>
__device__ __forceinline__ void quant1(float (&m)[32], const float (&sn)[8], const float (&inv)[8],
                                       const float* R, uint32_t (&w)[8], int lane, uint32_t n_valid,
                                       TileStats& ts) {
  constexpr int qmax = (1 << (B - 1)) - 1;
#pragma unroll
  for (int n = 0; n < 32; ++n) {
    const int i = n >> 2;
    const float t = (m[n] * inv[i]) * static_cast<float>(qmax);
    int q = static_cast<int>(__builtin_rintf(t));
    q = min(max(q, -qmax), qmax);
    uint32_t u = static_cast<uint32_t>(q + qmax);
    if (TAIL && !is_valid(n, lane, n_valid)) u = 0;
    insert<B>(w, n, u);
    float mq = sn[i] * R[u];
    if (STATS) {
      if (TAIL && !is_valid(n, lane, n_valid)) mq = 0.0f;
      const float d = m[n] - mq;
      ts.m_sum += m[n];
      ts.m_sq += m[n] * m[n];
      ts.m_err += d * d;
    }
    m[n] = mq;
  }
}

// Logarithmic quantization of v: the code is the number of thresholds at or below
// rho = v/blockmax, found with one bucket lookup and one compare on the bit pattern of rho.
template <int B, bool STATS, bool TAIL>
__device__ __forceinline__ void quant2(float (&v)[32], const float (&sn)[8], const float (&inv)[8],
                                       const float* L, const uint2* VQ, uint32_t (&w)[8], int lane,
                                       uint32_t n_valid, TileStats& ts) {
#pragma unroll
  for (int n = 0; n < 32; ++n) {
    const int i = n >> 2;
    const float rho = v[n] * inv[i];
    const uint32_t bits = f2u(rho);
    const uint32_t idx = min(kVqTop - (bits >> kVqShift), static_cast<uint32_t>(kVqBuckets - 1));
    const uint2 e = VQ[idx];
    uint32_t c = e.y + (bits >= e.x ? 1u : 0u);
    if (TAIL && !is_valid(n, lane, n_valid)) c = 0;
    insert<B>(w, n, c);
    float vq = sn[i] * L[c];
    if (STATS) {
      if (TAIL && !is_valid(n, lane, n_valid)) vq = 0.0f;
      const float d = v[n] - vq;
      ts.v_sum += v[n];
      ts.v_sq += v[n] * v[n];
      ts.v_err += d * d;
    }
    v[n] = vq;
  }
}

#define STQ_SWITCH_BITS(bits, CALL)            \
  switch (bits) {                              \
    case 2: { constexpr int B = 2; CALL; } break; \
    case 3: { constexpr int B = 3; CALL; } break; \
    case 4: { constexpr int B = 4; CALL; } break; \
    case 5: { constexpr int B = 5; CALL; } break; \
    case 6: { constexpr int B = 6; CALL; } break; \
    case 7: { constexpr int B = 7; CALL; } break; \
    default: { constexpr int B = 8; CALL; } break; \
  }

// ------------------------------------------------------------------ one tile
template <bool BF16, bool STATS, bool TAIL>
__device__ __forceinline__ void process_tile(const TensorDesc& d, uint32_t tile, uint32_t n_valid,
                                             const StepArgs& a, const uint32_t* lds, uint32_t* ws,
                                             int lane, LaneStats& acc) {
  const uint32_t lgK = a.lgK;
  const uint32_t bm = d.bm, bv = d.bv;
  const size_t e0 = static_cast<size_t>(tile) * kTile;
  float* P = d.param + e0;
  uint32_t* CM = d.m_codes + static_cast<size_t>(tile) * 64u * bm;
  uint32_t* CV = d.v_codes + static_cast<size_t>(tile) * 64u * bv;
  const size_t sbase = static_cast<size_t>(tile) << (11 - lgK);  // scales per tile = 2048/K

  // ---- loads -------------------------------------------------------------
  // Lane L = (value vL = L&15, lane group qL = L>>4) is the owner of one (state, row) pair's
  // block scale: state = vL>>3, row = vL&7, block within the row = qL >> (lgK-6).
  const int vL = lane & 15, qL = lane >> 4;
  const uint32_t sidx = (static_cast<uint32_t>(vL & 7) << (8 - lgK)) + (static_cast<uint32_t>(qL) >> (lgK - 6));
  float* SC = (vL >> 3) ? d.v_scales : d.m_scales;
  const float sc_old = SC[sbase + sidx];

  uint32_t wm[8], wv[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) if (p < static_cast<int>(bm)) wm[p] = CM[p * 64 + lane];
#pragma unroll
  for (int p = 0; p < 8; ++p) if (p < static_cast<int>(bv)) wv[p] = CV[p * 64 + lane];

  float g[32];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (!TAIL) {
      if (BF16) {
        const uint2 r = reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(d.grad) + e0 + 256 * i)[lane];
        g[4 * i + 0] = u2f(r.x << 16); g[4 * i + 1] = u2f(r.x & 0xFFFF0000u);
        g[4 * i + 2] = u2f(r.y << 16); g[4 * i + 3] = u2f(r.y & 0xFFFF0000u);
      } else {
        const float4 r = reinterpret_cast<const float4*>(static_cast<const float*>(d.grad) + e0 + 256 * i)[lane];
        g[4 * i + 0] = r.x; g[4 * i + 1] = r.y; g[4 * i + 2] = r.z; g[4 * i + 3] = r.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int n = 4 * i + e;
        float x = 0.0f;
        if (is_valid(n, lane, n_valid)) {
          const size_t idx = e0 + 256 * i + 4 * lane + e;
          x = BF16 ? u2f(static_cast<uint32_t>(static_cast<const uint16_t*>(d.grad)[idx]) << 16)
                   : static_cast<const float*>(d.grad)[idx];
        }
        g[n] = x;
      }
    }
  }

  // old scales to every lane that needs them: lane j reads the 16 values of its lane group
  float* wsf = reinterpret_cast<float*>(ws);
  float* X = wsf;                  // [16][XS]
  float* SO = wsf + 16 * XS;       // [64] old scales by owner lane
  float* SN = SO + 64;             // [64] new scales
  float* SI = SN + 64;             // [64] reciprocals of the new scales
  SO[lane] = sc_old;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float som[8], sov[8];
  {
    const float4* s4 = reinterpret_cast<const float4*>(SO + (lane >> 4) * 16);
    const float4 a0 = s4[0], a1 = s4[1], a2 = s4[2], a3 = s4[3];
    som[0] = a0.x; som[1] = a0.y; som[2] = a0.z; som[3] = a0.w;
    som[4] = a1.x; som[5] = a1.y; som[6] = a1.z; som[7] = a1.w;
    sov[0] = a2.x; sov[1] = a2.y; sov[2] = a2.z; sov[3] = a2.w;
    sov[4] = a3.x; sov[5] = a3.y; sov[6] = a3.z; sov[7] = a3.w;
  }

  TileStats ts;
  if (STATS) {
#pragma unroll
    for (int n = 0; n < 32; ++n) {
      ts.g_sum += g[n];
      ts.g_abs += fabsf(g[n]);
      ts.g_sq += g[n] * g[n];
      ts.g_max = fmaxf(ts.g_max, fabsf(g[n]));
    }
  }

  // ---- moments -----------------------------------------------------------
  const float* ldsf = reinterpret_cast<const float*>(lds);
  float m[32], v[32];
  STQ_SWITCH_BITS(bm, (moment1<B>(wm, ldsf + kTabROff + (1 << B) - 4, som, a.beta1, a.omb1, g, m)));
  STQ_SWITCH_BITS(bv, (moment2<B>(wv, ldsf + kTabLOff + (1 << B) - 4, sov, a.beta2, a.omb2, g, v)));
  if (TAIL) {
#pragma unroll
    for (int n = 0; n < 32; ++n)
      if (!is_valid(n, lane, n_valid)) { m[n] = 0.0f; v[n] = 0.0f; }
  }

  // ---- block maxima: lane partials -> LDS transpose -> one owner lane per (state,row,block)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float pm = fmaxf(fmaxf(fabsf(m[4 * i]), fabsf(m[4 * i + 1])), fmaxf(fabsf(m[4 * i + 2]), fabsf(m[4 * i + 3])));
    const float pv = fmaxf(fmaxf(v[4 * i], v[4 * i + 1]), fmaxf(v[4 * i + 2], v[4 * i + 3]));
    X[i * XS + lane] = pm;
    X[(8 + i) * XS + lane] = pv;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float r = 0.0f;
  {
    const float4* x4 = reinterpret_cast<const float4*>(X + vL * XS + qL * 16);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float4 t = x4[k];
      r = fmaxf(r, fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w)));
    }
  }
  if (lgK >= 7) r = fmaxf(r, __shfl_xor(r, 16, 64));
  if (lgK == 8) r = fmaxf(r, __shfl_xor(r, 32, 64));
  if (STATS) {
    if (vL < 8) ts.m_max = r; else ts.v_max = r;
  }
  // a block whose maximum is below the smallest normal number is stored as all-zero
  const float sc_new = (r < FLT_MIN) ? 0.0f : r;
  const float sc_inv = (sc_new > 0.0f) ? 1.0f / sc_new : 0.0f;
  SN[lane] = sc_new;
  SI[lane] = sc_inv;
  if ((static_cast<uint32_t>(qL) & ((1u << (lgK - 6)) - 1u)) == 0u) SC[sbase + sidx] = sc_new;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float snm[8], snv[8], sim[8], siv[8];
  {
    const float4* s4 = reinterpret_cast<const float4*>(SN + (lane >> 4) * 16);
    const float4* i4 = reinterpret_cast<const float4*>(SI + (lane >> 4) * 16);
    const float4 a0 = s4[0], a1 = s4[1], a2 = s4[2], a3 = s4[3];
    const float4 b0 = i4[0], b1 = i4[1], b2 = i4[2], b3 = i4[3];
    snm[0] = a0.x; snm[1] = a0.y; snm[2] = a0.z; snm[3] = a0.w;
    snm[4] = a1.x; snm[5] = a1.y; snm[6] = a1.z; snm[7] = a1.w;
    snv[0] = a2.x; snv[1] = a2.y; snv[2] = a2.z; snv[3] = a2.w;
    snv[4] = a3.x; snv[5] = a3.y; snv[6] = a3.z; snv[7] = a3.w;
    sim[0] = b0.x; sim[1] = b0.y; sim[2] = b0.z; sim[3] = b0.w;
    sim[4] = b1.x; sim[5] = b1.y; sim[6] = b1.z; sim[7] = b1.w;
    siv[0] = b2.x; siv[1] = b2.y; siv[2] = b2.z; siv[3] = b2.w;
    siv[4] = b3.x; siv[5] = b3.y; siv[6] = b3.z; siv[7] = b3.w;
  }

  // ---- quantize, pack, and replace m, v by their quantized values ----------
  STQ_SWITCH_BITS(bm, (quant1<B, STATS, TAIL>(m, snm, sim, ldsf + kTabROff + (1 << B) - 4, wm, lane, n_valid, ts)));
  STQ_SWITCH_BITS(bv, (quant2<B, STATS, TAIL>(v, snv, siv, ldsf + kTabLOff + (1 << B) - 4,
                                              reinterpret_cast<const uint2*>(lds + kTabVqOff) + (B - 2) * kVqBuckets,
                                              wv, lane, n_valid, ts)));
#pragma unroll
  for (int p = 0; p < 8; ++p) if (p < static_cast<int>(bm)) CM[p * 64 + lane] = wm[p];
#pragma unroll
  for (int p = 0; p < 8; ++p) if (p < static_cast<int>(bv)) CV[p * 64 + lane] = wv[p];

  // ---- bias correction of the quantized moments and the parameter update ---
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float th[4];
    if (!TAIL) {
      const float4 t = reinterpret_cast<const float4*>(P + 256 * i)[lane];
      th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        th[e] = is_valid(4 * i + e, lane, n_valid) ? P[256 * i + 4 * lane + e] : 0.0f;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = 4 * i + e;
      const float mt = m[n] * a.ibc1;
      const float vt = v[n] * a.ibc2;
      const float den = __builtin_sqrtf(vt) + a.eps;
      const float ratio = mt / den;
      const float upd = a.lr * ratio;
      const float dec = th[e] * a.decay;
      th[e] = dec - upd;
    }
    if (!TAIL) {
      reinterpret_cast<float4*>(P + 256 * i)[lane] = make_float4(th[0], th[1], th[2], th[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (is_valid(4 * i + e, lane, n_valid)) P[256 * i + 4 * lane + e] = th[e];
    }
  }

  if (STATS) {
    acc.g_sum += ts.g_sum; acc.g_abs += ts.g_abs; acc.g_sq += ts.g_sq;
    acc.m_sum += ts.m_sum; acc.m_sq += ts.m_sq; acc.m_err += ts.m_err;
    acc.v_sum += ts.v_sum; acc.v_sq += ts.v_sq; acc.v_err += ts.v_err;
    acc.g_max = fmaxf(acc.g_max, ts.g_max);
    acc.m_max = fmaxf(acc.m_max, ts.m_max);
    acc.v_max = fmaxf(acc.v_max, ts.v_max);
  }
}

// -------------------------------------------------------------- step kernel
// Every wavefront takes a contiguous range of the launch-wide tile order, so it crosses few
// tensor boundaries and flushes its statistics once per tensor it touched.
template <bool BF16, bool STATS>
__global__ __launch_bounds__(256, 2) void step_kernel(const StepArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsWords];
  for (int i = threadIdx.x; i < kTabWords; i += 256) lds[i] = a.tables[i];
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t* ws = lds + kTabWords + wave * kWaveScratch;
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * kWavesPerGroup;
  const uint64_t gw = static_cast<uint64_t>(blockIdx.x) * kWavesPerGroup + wave;
  uint32_t t = static_cast<uint32_t>(a.total_tiles * gw / n_waves);
  const uint32_t t_end = static_cast<uint32_t>(a.total_tiles * (gw + 1) / n_waves);
  if (t >= t_end) return;

  // tensor holding tile t: last l with tile_begin <= t
  uint32_t lo = 0, hi = a.n_tensors - 1;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) >> 1;
    if (a.desc[mid].tile_begin <= t) lo = mid; else hi = mid - 1;
  }
  uint32_t l = __builtin_amdgcn_readfirstlane(lo);

  while (t < t_end) {
    const TensorDesc d = a.desc[l];
    const uint32_t stop = min(t_end, d.tile_begin + d.n_tiles);
    LaneStats acc;
    if (STATS) acc.clear();
    for (; t < stop; ++t) {
      const uint32_t tile = t - d.tile_begin;
      const uint64_t left = d.numel - static_cast<uint64_t>(tile) * kTile;
      if (left >= static_cast<uint64_t>(kTile)) {
        process_tile<BF16, STATS, false>(d, tile, kTile, a, lds, ws, lane, acc);
      } else {
        process_tile<BF16, STATS, true>(d, tile, static_cast<uint32_t>(left), a, lds, ws, lane, acc);
      }
    }
    if (STATS) flush_stats(acc, a.stats + static_cast<size_t>(l) * kStatSlots, lane);
    ++l;
  }
}

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

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, uint64_t words) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < words) p[i] = 0u;
}

}  // namespace

// -------------------------------------------------------------------- launchers
int launch_step(const StepArgs& a, bool grad_bf16, bool want_stats, uint32_t groups, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(groups), block(256);
  if (grad_bf16) {
    if (want_stats) hipLaunchKernelGGL((step_kernel<true, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((step_kernel<true, false>), grid, block, 0, s, a);
  } else {
    if (want_stats) hipLaunchKernelGGL((step_kernel<false, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((step_kernel<false, false>), grid, block, 0, s, a);
  }
  return static_cast<int>(hipGetLastError());
}

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

int launch_fill_zero(uint32_t* p, uint64_t words, void* stream) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<uint32_t>((words + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), p, words);
  return static_cast<int>(hipGetLastError());
}

}  // namespace stq
