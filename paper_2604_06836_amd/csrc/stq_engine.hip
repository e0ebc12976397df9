// Device-resident precision loop: Algorithm 1's periodic body (layer statistics -> global EMAs ->
// score -> Map; Eq. 2, 3, 4, 7, 8 and Section 3.4 of the paper) as one small kernel that reads the
// accumulators the step kernel filled and rewrites the device-resident tensor table for the next
// step, plus the host calls that enqueue the loop.  Nothing here copies back or waits, except
// stq_engine_read.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "stq_host.h"

using namespace stq;

namespace {

constexpr uint32_t kMaxThr = 15;
constexpr int kPlanThreads = 1024;
constexpr uint32_t kPlanLdsLayers = 1024;  // the factors of this many layers are summed from LDS, the rest from global memory

struct PlanCfg {  // the decision's parameters, by value
  double alpha, phi, eps, v_offset;
  double thr[kMaxThr];
  uint32_t n_thr, flags;
  uint8_t bits[kMaxThr + 1];
};

struct PlanArgs {
  TensorDesc* desc;
  uint32_t n;
  uint32_t decide;   // 0: only adopt what the last step wrote
  double* stats;     // [n][kStatSlots], cleared here after use
  double* fac;       // [n][3] scratch: n_l, r_l, v_l
  double* ema;       // n_ema, r_ema, v_ema
  double* score;     // [n]
  uint32_t** spare;  // [n][2]: the code buffer of each state that is not in use
  double log_s;      // log2 of the temporal factor S_t (Eq. 7), from the host
  PlanCfg cfg;
};

// Map: a step function of the score.  A score equal to a threshold takes the higher width.
__device__ uint32_t map_width(double score, const PlanCfg& c) {
  uint32_t above = 0;
  for (uint32_t i = 0; i < c.n_thr; ++i) above += (c.thr[i] <= score) ? 1u : 0u;
  return c.bits[above];
}

// One workgroup.  (1) every tensor adopts what the step just wrote (its new width and buffer become
// the stored ones); (2) with `decide`: per-layer factors in parallel, their sums over the layers by
// one lane each in layer order (the order of the host-side decision, so the EMAs agree to the bit
// given equal statistics), then score and Map in parallel; the new widths and destinations go into
// the table for the next step.
__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const PlanArgs a) {
  __shared__ double sh_ema[3];
  __shared__ double sh_fac[3][kPlanLdsLayers];
  const uint32_t tid = threadIdx.x;
  for (uint32_t l = tid; l < a.n; l += kPlanThreads) {
    TensorDesc& d = a.desc[l];
    if (d.m_out != d.m_codes) { a.spare[2 * l] = d.m_codes; d.m_codes = d.m_out; }
    if (d.v_out != d.v_codes) { a.spare[2 * l + 1] = d.v_codes; d.v_codes = d.v_out; }
    d.bm = d.bm_out;
    d.bv = d.bv_out;
    if (!a.decide) continue;
    double* s = a.stats + static_cast<size_t>(l) * kStatSlots;
    const double cnt = static_cast<double>(d.numel);
    const double mean_sq = s[kGSqSum] / cnt;    // v_l   (Eq. 8)
    const double mean_abs = s[kGAbsSum] / cnt;
    const double rms = sqrt(mean_sq);           // n_l   (Eq. 2)
    double var;
    if (a.cfg.flags & STQ_DECIDE_R_ALG1) {
      const double mean = s[kGSum] / cnt;
      var = mean_sq - mean * mean;              // sigma(g)^2, Algorithm 1's form
    } else {
      var = mean_sq - mean_abs * mean_abs;      // sigma(|g|)^2, Eq. 3
    }
    if (var < 0.0) var = 0.0;
    const double cv = sqrt(var) / (mean_abs + a.cfg.eps);  // r_l
    a.fac[3 * l] = rms; a.fac[3 * l + 1] = cv; a.fac[3 * l + 2] = mean_sq;
    if (l < kPlanLdsLayers) { sh_fac[0][l] = rms; sh_fac[1][l] = cv; sh_fac[2][l] = mean_sq; }
    for (int k = 0; k < kStatSlots; ++k) s[k] = 0.0;
  }
  if (!a.decide) return;
  __threadfence_block();
  __syncthreads();
  if (tid < 3) {
    double sum = 0.0;  // in layer order, as the host-side decision sums
    const uint32_t in_lds = a.n < kPlanLdsLayers ? a.n : kPlanLdsLayers;
    for (uint32_t l = 0; l < in_lds; ++l) sum += sh_fac[tid][l];
    for (uint32_t l = in_lds; l < a.n; ++l) sum += a.fac[3 * l + tid];
    const double al = a.cfg.alpha, inv_n = 1.0 / static_cast<double>(a.n);
    const double e = al * (sum * inv_n) + (1.0 - al) * a.ema[tid];  // Eq. 4
    a.ema[tid] = e;
    sh_ema[tid] = e;
  }
  __syncthreads();
  const double n_ema = sh_ema[0], r_ema = sh_ema[1], v_ema = sh_ema[2];
  for (uint32_t l = tid; l < a.n; l += kPlanThreads) {
    double score = a.cfg.phi;
    if (!(a.cfg.flags & STQ_DECIDE_NO_DUAL))
      score += log2(a.fac[3 * l + 1] / (r_ema + a.cfg.eps)) + log2(a.fac[3 * l] / (n_ema + a.cfg.eps));
    if (!(a.cfg.flags & STQ_DECIDE_NO_TEMPORAL)) score += a.log_s;
    if (!(a.cfg.flags & STQ_DECIDE_NO_SPATIAL)) score += log2(a.fac[3 * l + 2] / (v_ema + a.cfg.eps));
    a.score[l] = score;
    TensorDesc& d = a.desc[l];
    const uint32_t bm = map_width(score, a.cfg), bv = map_width(score + a.cfg.v_offset, a.cfg);
    d.bm_out = bm;
    d.bv_out = bv;
    d.m_out = (bm != d.bm) ? a.spare[2 * l] : d.m_codes;
    d.v_out = (bv != d.bv) ? a.spare[2 * l + 1] : d.v_codes;
  }
}

__global__ void set_grads_kernel(TensorDesc* desc, const void* const* grads, uint32_t n) {
  const uint32_t l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l < n) desc[l].grad = grads[l];
}

}  // namespace

struct stq_engine {
  stq_ctx* ctx = nullptr;
  uint32_t n = 0, total_tiles = 0, block = 0;
  bool wide = false;      // some state may be 16 or 32 bits wide: the kernel variant that handles them
  bool quarters_ok = true;  // every width the loop can take is a multiple of 4 bits
  uint32_t v_widths = 0;    // bit b set: a second moment can be quantized at width b (initial plan or the ladder)
  bool alg1_order = false;  // decide from a pass over the gradients before the step, as Algorithm 1 is written
  bool stepped = false;     // a step has been enqueued
  uint32_t capacity_bits = 0;
  std::vector<TensorDesc> h_desc;   // the table as created (for stq_engine_set_next, before the first step)
  std::vector<uint32_t*> h_spare;
  bool pending = false;   // the table holds widths/destinations that differ from the stored ones
  double tau = 0.0;
  PlanCfg cfg;
  TensorDesc* d_desc = nullptr;
  double* d_stats = nullptr;
  double* d_fac = nullptr;
  double* d_ema = nullptr;
  double* d_score = nullptr;
  uint32_t** d_spare = nullptr;
  const void** d_grads = nullptr;
  const void** h_grads[kRing] = {};  // pinned
  hipEvent_t grads_done[kRing] = {};
  int grads_pos = 0;
  void* h_read = nullptr;  // pinned staging of stq_engine_read
};

extern "C" {

int stq_engine_destroy(stq_engine* e) {
  if (!e) return STQ_EINVAL;
  DeviceGuard g(e->ctx->device);
  (void)hipDeviceSynchronize();
  if (e->d_desc) (void)hipFree(e->d_desc);
  if (e->d_stats) (void)hipFree(e->d_stats);
  if (e->d_fac) (void)hipFree(e->d_fac);
  if (e->d_ema) (void)hipFree(e->d_ema);
  if (e->d_score) (void)hipFree(e->d_score);
  if (e->d_spare) (void)hipFree(e->d_spare);
  if (e->d_grads) (void)hipFree(e->d_grads);
  for (int k = 0; k < kRing; ++k) {
    if (e->h_grads[k]) (void)hipHostFree(e->h_grads[k]);
    if (e->grads_done[k]) (void)hipEventDestroy(e->grads_done[k]);
  }
  if (e->h_read) (void)hipHostFree(e->h_read);
  delete e;
  return STQ_OK;
}

int stq_engine_create(stq_ctx* ctx, stq_engine** out, const stq_tensor* tensors, const stq_codes* second,
                      uint32_t n, const stq_bits* initial_plan, uint32_t capacity_bits, uint32_t block,
                      const stq_decide_cfg* cfg, const stq_decide_state* ema, uint32_t flags, void* stream) {
  if (!out) return STQ_EINVAL;
  *out = nullptr;
  if (flags & ~STQ_ENGINE_ALG1_ORDER) return STQ_EINVAL;
  if (!ctx || !tensors || !second || !initial_plan || !cfg) return STQ_EINVAL;
  if (cfg->n_thr > kMaxThr || (cfg->n_thr > 0 && !cfg->thr) || !cfg->bits) return STQ_EINVAL;
  if (!(cfg->tau > 0.0) || !(cfg->alpha >= 0.0 && cfg->alpha <= 1.0)) return STQ_EINVAL;
  if (int err = check_bits_stored(capacity_bits)) return err;
  std::vector<TensorDesc> descs;
  uint32_t total = 0;
  if (int err = build_descs(ctx, tensors, n, initial_plan, block, true, descs, &total)) return err;
  bool wide = false, quarters_ok = true;
  uint32_t v_widths = 0;
  for (uint32_t i = 0; i <= cfg->n_thr; ++i) {
    if (int err = check_bits_stored(cfg->bits[i])) return err;
    if (cfg->bits[i] > capacity_bits) return STQ_EINVAL;
    wide = wide || is_wide(cfg->bits[i]);
    quarters_ok = quarters_ok && (cfg->bits[i] & 3u) == 0;
    if (cfg->bits[i] <= 8) v_widths |= 1u << cfg->bits[i];
  }
  std::vector<uint32_t*> spare(2 * static_cast<size_t>(n));
  for (uint32_t l = 0; l < n; ++l) {
    if (initial_plan[l].m_bits > capacity_bits || initial_plan[l].v_bits > capacity_bits) return STQ_EINVAL;
    wide = wide || is_wide(initial_plan[l].m_bits) || is_wide(initial_plan[l].v_bits);
    quarters_ok = quarters_ok && ((initial_plan[l].m_bits | initial_plan[l].v_bits) & 3u) == 0;
    if (initial_plan[l].v_bits <= 8) v_widths |= 1u << initial_plan[l].v_bits;
    // the second buffers: distinct from the first over the whole capacity
    const uintptr_t span = static_cast<uintptr_t>(descs[l].n_tiles) * 256 * capacity_bits;
    const void* first[2] = {tensors[l].m_codes, tensors[l].v_codes};
    void* sec[2] = {second[l].m_codes, second[l].v_codes};
    for (int st = 0; st < 2; ++st) {
      if (!sec[st]) return STQ_EINVAL;
      if (!aligned(sec[st], 256)) return STQ_EALIGN;
      const uintptr_t a0 = reinterpret_cast<uintptr_t>(first[st]), b0 = reinterpret_cast<uintptr_t>(sec[st]);
      if (a0 < b0 + span && b0 < a0 + span) return STQ_EINVAL;
      spare[2 * l + st] = static_cast<uint32_t*>(sec[st]);
    }
  }

  stq_engine* e = new (std::nothrow) stq_engine();
  if (!e) return STQ_EINVAL;
  e->ctx = ctx;
  e->n = n;
  e->total_tiles = total;
  e->block = block;
  e->wide = wide;
  e->quarters_ok = quarters_ok;
  e->v_widths = v_widths;
  e->capacity_bits = capacity_bits;
  e->h_desc = descs;
  e->h_spare = spare;
  e->alg1_order = (flags & STQ_ENGINE_ALG1_ORDER) != 0;
  e->tau = cfg->tau;
  std::memset(&e->cfg, 0, sizeof(e->cfg));
  e->cfg.alpha = cfg->alpha; e->cfg.phi = cfg->phi; e->cfg.eps = cfg->eps; e->cfg.v_offset = cfg->v_offset;
  e->cfg.n_thr = cfg->n_thr; e->cfg.flags = cfg->flags;
  for (uint32_t i = 0; i < cfg->n_thr; ++i) e->cfg.thr[i] = cfg->thr[i];
  for (uint32_t i = 0; i <= cfg->n_thr; ++i) e->cfg.bits[i] = cfg->bits[i];

  DeviceGuard g(ctx->device);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t read_bytes = sizeof(TensorDesc) * n + sizeof(double) * (n + 3);
  bool ok = g.ok;
  ok = ok && hipMalloc(&e->d_desc, sizeof(TensorDesc) * n) == hipSuccess;
  ok = ok && hipMalloc(&e->d_stats, sizeof(double) * kStatSlots * n) == hipSuccess;
  ok = ok && hipMalloc(&e->d_fac, sizeof(double) * 3 * n) == hipSuccess;
  ok = ok && hipMalloc(&e->d_ema, sizeof(double) * 3) == hipSuccess;
  ok = ok && hipMalloc(&e->d_score, sizeof(double) * n) == hipSuccess;
  ok = ok && hipMalloc(&e->d_spare, sizeof(uint32_t*) * 2 * n) == hipSuccess;
  ok = ok && hipMalloc(&e->d_grads, sizeof(void*) * n) == hipSuccess;
  for (int k = 0; k < kRing && ok; ++k) {
    ok = ok && hipHostMalloc(&e->h_grads[k], sizeof(void*) * n, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&e->grads_done[k], hipEventDisableTiming) == hipSuccess;
  }
  ok = ok && hipHostMalloc(&e->h_read, read_bytes, hipHostMallocDefault) == hipSuccess;
  // the uploads come from pageable host memory, so each call returns only after its source was read
  const double ema0[3] = {ema ? ema->n_ema : 0.0, ema ? ema->r_ema : 0.0, ema ? ema->v_ema : 0.0};
  ok = ok && hipMemcpyAsync(e->d_desc, descs.data(), sizeof(TensorDesc) * n, hipMemcpyHostToDevice, s) == hipSuccess;
  ok = ok && hipMemcpyAsync(e->d_spare, spare.data(), sizeof(uint32_t*) * 2 * n, hipMemcpyHostToDevice, s) == hipSuccess;
  ok = ok && hipMemcpyAsync(e->d_ema, ema0, sizeof(ema0), hipMemcpyHostToDevice, s) == hipSuccess;
  ok = ok && launch_fill_zero(reinterpret_cast<uint32_t*>(e->d_stats), sizeof(double) * kStatSlots * n / 4, stream) == 0;
  ok = ok && launch_fill_zero(reinterpret_cast<uint32_t*>(e->d_score), sizeof(double) * n / 4, stream) == 0;
  ok = ok && hipStreamSynchronize(s) == hipSuccess;
  if (!ok) { stq_engine_destroy(e); return STQ_EHIP; }
  *out = e;
  return STQ_OK;
}

int stq_engine_set_next(stq_engine* e, const stq_bits* next, void* stream) {
  if (!e || !next) return STQ_EINVAL;
  if (e->stepped || e->alg1_order) return STQ_ESTATE;
  bool pending = false;
  std::vector<TensorDesc> descs = e->h_desc;
  for (uint32_t l = 0; l < e->n; ++l) {
    TensorDesc& d = descs[l];
    const uint32_t w[2] = {next[l].m_bits, next[l].v_bits};
    for (uint32_t b : w) {
      if (int err = check_bits_stored(b)) return err;
      bool on_ladder = false;  // a decision of this loop can only have chosen widths of its ladder
      for (uint32_t i = 0; i <= e->cfg.n_thr; ++i) on_ladder = on_ladder || e->cfg.bits[i] == b;
      if (!on_ladder || b > e->capacity_bits) return STQ_EINVAL;
    }
    d.bm_out = w[0];
    d.bv_out = w[1];
    d.m_out = w[0] != d.bm ? e->h_spare[2 * l] : d.m_codes;
    d.v_out = w[1] != d.bv ? e->h_spare[2 * l + 1] : d.v_codes;
    pending = pending || w[0] != d.bm || w[1] != d.bv;
  }
  DeviceGuard g(e->ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // from pageable host memory: the call returns only after its source was read
  if (hipMemcpyAsync(e->d_desc, descs.data(), sizeof(TensorDesc) * e->n, hipMemcpyHostToDevice, s) != hipSuccess) return STQ_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return STQ_EHIP;
  e->pending = pending;
  return STQ_OK;
}

int stq_engine_step(stq_engine* e, const stq_hparams* hp, uint32_t update_every, const void* const* grads,
                    void* stream) {
  if (!e) return STQ_EINVAL;
  if (int err = check_hparams(hp)) return err;
  if (hp->block != e->block) return STQ_EBLOCK;
  if (grads)
    for (uint32_t l = 0; l < e->n; ++l) {
      if (!grads[l]) return STQ_EINVAL;
      if (!aligned(grads[l], 16)) return STQ_EALIGN;
    }
  DeviceGuard g(e->ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (grads) {
    const int k = e->grads_pos;
    e->grads_pos = (k + 1) % kRing;
    if (int err = wait_slot_free(e->grads_done[k])) return err;
    std::memcpy(e->h_grads[k], grads, sizeof(void*) * e->n);
    if (hipMemcpyAsync(e->d_grads, e->h_grads[k], sizeof(void*) * e->n, hipMemcpyHostToDevice, s) != hipSuccess)
      return STQ_EHIP;
    if (hipEventRecord(e->grads_done[k], s) != hipSuccess) return STQ_EHIP;
    hipLaunchKernelGGL(set_grads_kernel, dim3((e->n + 255) / 256), dim3(256), 0, s, e->d_desc, e->d_grads, e->n);
    if (hipGetLastError() != hipSuccess) return STQ_EHIP;
  }
  const bool due = stq_decide_due(hp->step, update_every) != 0;
  e->stepped = true;
  stq_hparams h = *hp;
  auto plan = [&](bool decide) -> int {
    PlanArgs a;
    a.desc = e->d_desc;
    a.n = e->n;
    a.decide = decide ? 1u : 0u;
    a.stats = e->d_stats;
    a.fac = e->d_fac;
    a.ema = e->d_ema;
    a.score = e->d_score;
    a.spare = e->d_spare;
    // temporal annealing factor, Eq. 7
    a.log_s = std::log2(1.0 + 1.0 / std::cosh(static_cast<double>(hp->step) / e->tau));
    a.cfg = e->cfg;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, a);
    return hipGetLastError() == hipSuccess ? STQ_OK : STQ_EHIP;
  };
  if (e->alg1_order) {
    // Algorithm 1 as written: statistics of g_t and Map first, then this step's layer loop at the new widths
    h.flags = 0u;
    if (due) {
      if (launch_grad_stats(e->d_desc, e->n, e->total_tiles, e->d_stats, hp->grad_dtype == 1,
                            grad_stats_groups(e->ctx->n_cu, e->total_tiles), stream) != 0)
        return STQ_EHIP;
      if (int err = plan(true)) return err;
    }
    const int mode = e->wide ? 2 : (due ? 1 : 0);
    if (int err = launch_table(e->ctx, e->d_desc, e->n, e->total_tiles, e->d_stats, &h, mode, e->quarters_ok, e->v_widths, stream)) return err;
    if (due) return plan(false);  // the states now are what the step wrote
    return STQ_OK;
  }
  // by-product order: the step gathers the statistics, the decision takes effect in the next step
  h.flags = due ? STQ_FLAG_STATS_GRAD : 0u;  // the decision reads the gradient's sums only
  // kernel variant: the widths in the table differ from the stored ones only in the step after a decision
  const int mode = e->wide ? 2 : (e->pending ? 1 : 0);
  if (int err = launch_table(e->ctx, e->d_desc, e->n, e->total_tiles, e->d_stats, &h, mode, e->quarters_ok, e->v_widths, stream)) return err;
  if (due || e->pending) {
    if (int err = plan(due)) return err;
    e->pending = due;
  }
  return STQ_OK;
}

int stq_engine_read(stq_engine* e, stq_bits* stored, stq_bits* next, stq_codes* current, double* score,
                    stq_decide_state* ema, void* stream) {
  if (!e) return STQ_EINVAL;
  DeviceGuard g(e->ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint32_t n = e->n;
  TensorDesc* hd = static_cast<TensorDesc*>(e->h_read);
  double* hs = reinterpret_cast<double*>(hd + n);
  if (hipMemcpyAsync(hd, e->d_desc, sizeof(TensorDesc) * n, hipMemcpyDeviceToHost, s) != hipSuccess) return STQ_EHIP;
  if (hipMemcpyAsync(hs, e->d_score, sizeof(double) * n, hipMemcpyDeviceToHost, s) != hipSuccess) return STQ_EHIP;
  if (hipMemcpyAsync(hs + n, e->d_ema, sizeof(double) * 3, hipMemcpyDeviceToHost, s) != hipSuccess) return STQ_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return STQ_EHIP;
  for (uint32_t l = 0; l < n; ++l) {
    if (stored) { stored[l].m_bits = static_cast<uint8_t>(hd[l].bm); stored[l].v_bits = static_cast<uint8_t>(hd[l].bv); }
    if (next) { next[l].m_bits = static_cast<uint8_t>(hd[l].bm_out); next[l].v_bits = static_cast<uint8_t>(hd[l].bv_out); }
    if (current) { current[l].m_codes = hd[l].m_codes; current[l].v_codes = hd[l].v_codes; }
    if (score) score[l] = hs[l];
  }
  if (ema) { ema->n_ema = hs[n]; ema->r_ema = hs[n + 1]; ema->v_ema = hs[n + 2]; }
  return STQ_OK;
}

}  // extern "C"
