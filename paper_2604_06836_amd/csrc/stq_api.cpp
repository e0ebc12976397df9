// Host side of the C ABI declared in include/stq.h: argument checks, the device-resident
// tensor table, kernel launches, statistics read-back.  Compiled by hipcc (HIP runtime calls).
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "stq_host.h"
#include "stq_tables.h"

using namespace stq;

namespace stq {

int fill_descs(const stq_ctx* ctx, const stq_tensor* t, uint32_t n, const stq_bits* plan, uint32_t K,
               bool need_param_grad, TensorDesc* out, uint32_t* total_tiles) {
  if (!ctx || !t || !plan || n == 0 || n > ctx->max_tensors) return STQ_EINVAL;
  if (lg_block(K) < 0) return STQ_EBLOCK;
  uint64_t tiles = 0;
  for (uint32_t l = 0; l < n; ++l) {
    if (int e = check_bits_stored(plan[l].m_bits)) return e;
    if (int e = check_bits_stored(plan[l].v_bits)) return e;
    if (t[l].numel == 0) return STQ_EINVAL;
    if (!t[l].m_codes || !t[l].m_scales || !t[l].v_codes || !t[l].v_scales) return STQ_EINVAL;
    if (need_param_grad && (!t[l].param || !t[l].grad)) return STQ_EINVAL;
    if (!aligned(t[l].m_codes, 256) || !aligned(t[l].m_scales, 256) || !aligned(t[l].v_codes, 256) ||
        !aligned(t[l].v_scales, 256))
      return STQ_EALIGN;
    if (need_param_grad && (!aligned(t[l].param, 16) || !aligned(t[l].grad, 16))) return STQ_EALIGN;
    const uint64_t nt = (t[l].numel + kTile - 1) / kTile;
    if (tiles + nt > 0xFFFFFFFFull) return STQ_EINVAL;
    TensorDesc& d = out[l];
    d.param = static_cast<float*>(t[l].param);
    d.grad = t[l].grad;
    d.m_codes = static_cast<uint32_t*>(t[l].m_codes);
    d.m_scales = t[l].m_scales;
    d.v_codes = static_cast<uint32_t*>(t[l].v_codes);
    d.v_scales = t[l].v_scales;
    d.numel = t[l].numel;
    d.tile_begin = static_cast<uint32_t>(tiles);
    d.n_tiles = static_cast<uint32_t>(nt);
    d.bm = plan[l].m_bits;
    d.bv = plan[l].v_bits;
    d.m_out = d.m_codes;  // in place unless a caller redirects them
    d.v_out = d.v_codes;
    d.bm_out = d.bm;
    d.bv_out = d.bv;
    tiles += nt;
  }
  *total_tiles = static_cast<uint32_t>(tiles);
  return STQ_OK;
}

int build_descs(const stq_ctx* ctx, const stq_tensor* t, uint32_t n, const stq_bits* plan, uint32_t K,
                bool need_param_grad, std::vector<TensorDesc>& out, uint32_t* total_tiles) {
  if (!ctx || n == 0 || n > ctx->max_tensors) return STQ_EINVAL;
  out.resize(n);
  return fill_descs(ctx, t, n, plan, K, need_param_grad, out.data(), total_tiles);
}

}  // namespace stq

// ---------------------------------------------------------------- static scratch
// Device memory of stq_step_static, the entry point that allocates nothing: the tensor table its
// kernel reads.  One copy per GPU, held until the process ends.  In host code the array's name is only
// a stand-in for the symbol: the address that kernels and copies use comes from hipGetSymbolAddress,
// once per device (stq_init), and is kept in g_static_scratch.
namespace {

constexpr uint32_t kStaticMaxTensors = STQ_STATIC_MAX_TENSORS;
constexpr size_t kStaticTableBytes = sizeof(TensorDesc) * kStaticMaxTensors;
constexpr size_t kStaticScratchBytes = kStaticTableBytes + 256;  // the table, then the scheduling words
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices];  // per device, null until a context was created on it

// With `device` current: the address of that device's copy of `scratch`.
int static_scratch_address(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return STQ_EDEVICE;
  if (!g_static_scratch[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return STQ_EHIP;
    g_static_scratch[device] = p;
  }
  *out = g_static_scratch[device];
  return STQ_OK;
}

}  // namespace

extern "C" {

const char* stq_strerror(int code) {
  switch (code) {
    case STQ_OK: return "ok";
    case STQ_EINVAL: return "invalid argument";
    case STQ_EALIGN: return "misaligned device buffer";
    case STQ_EBITS: return "bit-width not one of 2..8 (or, for a stored state, 16 or 32)";
    case STQ_EBLOCK: return "block size must be 64, 128 or 256";
    case STQ_EDEVICE: return "device missing or not gfx950";
    case STQ_EHIP: return "HIP runtime error";
    case STQ_ESTATE: return "no statistics accumulated";
    case STQ_ELIMIT: return "more tensors than the static scratch of stq_step_static holds";
    default: return "unknown error";
  }
}

int stq_state_bytes(uint64_t numel, uint32_t block, uint32_t bits, uint64_t* code_bytes,
                    uint64_t* scale_bytes) {
  if (numel == 0 || (!code_bytes && !scale_bytes)) return STQ_EINVAL;
  if (lg_block(block) < 0) return STQ_EBLOCK;
  if (int e = check_bits_stored(bits)) return e;
  const uint64_t tiles = (numel + kTile - 1) / kTile;
  if (code_bytes) *code_bytes = tiles * 64ull * bits * 4ull;
  if (scale_bytes) *scale_bytes = tiles * (kTile / block) * 4ull;
  return STQ_OK;
}

int stq_table(int which, uint32_t bits, float* out, uint32_t n) {
  if (!out) return STQ_EINVAL;
  if (which == 0) {
    for (uint32_t j = 0; j < n && j < static_cast<uint32_t>(kGLen); ++j) out[j] = table_G(static_cast<int>(j));
    return kGLen;
  }
  if (int e = check_bits(bits)) return e;
  const int b = static_cast<int>(bits);
  int len;
  switch (which) {
    case 1: len = (1 << b) - 1; for (int u = 0; u < len && u < static_cast<int>(n); ++u) out[u] = table_R(b, u); break;
    case 2: len = (1 << b);     for (int c = 0; c < len && c < static_cast<int>(n); ++c) out[c] = table_L(b, c); break;
    case 3: len = (1 << b) - 1; for (int k = 0; k < len && k < static_cast<int>(n); ++k) out[k] = table_T(b, k); break;
    default: return STQ_EINVAL;
  }
  return len;
}

int stq_init(stq_ctx** out, int device, uint32_t max_tensors) {
  if (!out || max_tensors == 0 || max_tensors > (1u << 20)) return STQ_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return STQ_EDEVICE;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return STQ_EDEVICE;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return STQ_EDEVICE;
  std::vector<uint32_t> img;
  if (!build_table_image(img)) return STQ_EINVAL;

  stq_ctx* c = new (std::nothrow) stq_ctx();
  if (!c) return STQ_EINVAL;
  c->device = device;
  c->max_tensors = max_tensors;
  c->n_cu = static_cast<uint32_t>(prop.multiProcessorCount);
#ifdef STQ_TUNING_ENV  // measurement builds only: launch shape from the environment
  if (const char* e = std::getenv("STQ_GROUPS_PER_CU")) {
    const int v = std::atoi(e);
    if (v >= 1 && v <= 8) c->groups_per_cu = static_cast<uint32_t>(v);
  }
  if (const char* e = std::getenv("STQ_CHUNK")) {
    const long v = std::strtol(e, nullptr, 10);
    if (v >= 1 && v <= (1 << 20)) c->chunk_override = static_cast<uint32_t>(v);
  }
#endif
  DeviceGuard g(device);
  bool ok = g.ok;
  ok = ok && static_scratch_address(device, &c->static_scratch) == STQ_OK;
  ok = ok && hipMalloc(&c->d_tables, img.size() * 4) == hipSuccess;
  for (int k = 0; k < kDescTables && ok; ++k)
    ok = ok && hipMalloc(&c->d_desc[k], sizeof(TensorDesc) * max_tensors) == hipSuccess;
  ok = ok && hipMalloc(&c->d_stats, sizeof(double) * kStatSlots * max_tensors) == hipSuccess;
  ok = ok && hipMalloc(&c->d_sched, 256) == hipSuccess;
  ok = ok && hipMemset(c->d_sched, 0, 256) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_stats, sizeof(double) * kStatSlots * max_tensors, hipHostMallocDefault) == hipSuccess;
  for (int k = 0; k < kRing && ok; ++k) {
    ok = ok && hipHostMalloc(&c->h_stage[k], sizeof(TensorDesc) * max_tensors, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->stage_done[k], hipEventDisableTiming) == hipSuccess;
  }
  ok = ok && hipMemcpy(c->d_tables, img.data(), img.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
  // every conversion table of the re-pack: (state, old width, new width) -> 256 codes, one word each
  std::vector<uint32_t> luts(static_cast<size_t>(kRepackLuts) * 256);
  for (int st = 0; st < 2; ++st)
    for (int bo = kMinBits; bo <= kMaxBits; ++bo)
      for (int bn = kMinBits; bn <= kMaxBits; ++bn) {
        uint8_t one[256];
        build_repack_lut(st, bo, bn, one);
        uint32_t* dst = &luts[static_cast<size_t>(repack_lut_index(st, bo, bn)) * 256];
        for (int i = 0; i < 256; ++i) dst[i] = one[i];
      }
  ok = ok && hipMalloc(&c->d_luts, luts.size() * 4) == hipSuccess;
  ok = ok && hipMemcpy(c->d_luts, luts.data(), luts.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
  ok = ok && hipMalloc(&c->d_jobs, sizeof(RepackJob) * 2 * max_tensors) == hipSuccess;
  for (int k = 0; k < kRing && ok; ++k) {
    ok = ok && hipHostMalloc(&c->h_jobs[k], sizeof(RepackJob) * 2 * max_tensors, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->jobs_done[k], hipEventDisableTiming) == hipSuccess;
  }
  ok = ok && hipMemset(c->d_stats, 0, sizeof(double) * kStatSlots * max_tensors) == hipSuccess;
  ok = ok && hipDeviceSynchronize() == hipSuccess;
  if (!ok) { stq_destroy(c); return STQ_EHIP; }
  c->stat_count.assign(max_tensors, 0);
  c->descs.reserve(max_tensors);
  for (int k = 0; k < kDescTables; ++k) c->uploaded[k].reserve(max_tensors);
  *out = c;
  return STQ_OK;
}

int stq_set_schedule(stq_ctx* ctx, uint64_t ticket_min_tiles) {
  if (!ctx) return STQ_EINVAL;
  ctx->ticket_min_units = ticket_min_tiles ? ticket_min_tiles : kTicketMinUnits;
  return STQ_OK;
}

int stq_destroy(stq_ctx* c) {
  if (!c) return STQ_EINVAL;
  DeviceGuard g(c->device);
  (void)hipDeviceSynchronize();
  if (c->d_tables) (void)hipFree(c->d_tables);
  for (int k = 0; k < kDescTables; ++k)
    if (c->d_desc[k]) (void)hipFree(c->d_desc[k]);
  if (c->d_stats) (void)hipFree(c->d_stats);
  if (c->d_sched) (void)hipFree(c->d_sched);
  if (c->h_stats) (void)hipHostFree(c->h_stats);
  if (c->d_luts) (void)hipFree(c->d_luts);
  if (c->d_jobs) (void)hipFree(c->d_jobs);
  for (int k = 0; k < kRing; ++k) {
    if (c->h_jobs[k]) (void)hipHostFree(c->h_jobs[k]);
    if (c->jobs_done[k]) (void)hipEventDestroy(c->jobs_done[k]);
  }
  for (int k = 0; k < kRing; ++k) {
    if (c->h_stage[k]) (void)hipHostFree(c->h_stage[k]);
    if (c->stage_done[k]) (void)hipEventDestroy(c->stage_done[k]);
  }
  delete c;
  return STQ_OK;
}

int stq_zero_state(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, const stq_bits* plan,
                   uint32_t block, void* stream) {
  std::vector<TensorDesc> descs;
  uint32_t total = 0;
  if (int e = build_descs(ctx, tensors, n, plan, block, false, descs, &total)) return e;
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  for (uint32_t l = 0; l < n; ++l) {
    ZeroArgs a;
    a.m_codes = descs[l].m_codes; a.m_scales = descs[l].m_scales;
    a.v_codes = descs[l].v_codes; a.v_scales = descs[l].v_scales;
    a.numel = descs[l].numel; a.n_tiles = descs[l].n_tiles;
    a.bm = descs[l].bm; a.bv = descs[l].bv; a.scales_per_tile = kTile / block;
    if (launch_zero(a, stream) != 0) return STQ_EHIP;
  }
  return STQ_OK;
}

}  // extern "C"

namespace stq {

int check_hparams(const stq_hparams* hp) {
  if (!hp) return STQ_EINVAL;
  if (hp->step == 0 || hp->grad_dtype > 1) return STQ_EINVAL;
  // Adam's own preconditions: finite lr >= 0 and weight decay, 0 <= beta < 1, finite eps > 0
  if (!(hp->lr >= 0.0f) || !std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay)) return STQ_EINVAL;
  if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f)) return STQ_EINVAL;
  if (!(hp->eps > 0.0f) || !std::isfinite(hp->eps)) return STQ_EINVAL;
  if (lg_block(hp->block) < 0) return STQ_EBLOCK;
  return STQ_OK;
}

int launch_table(stq_ctx* ctx, const TensorDesc* d_desc, uint32_t n, uint32_t total, double* d_stats,
                 const stq_hparams* hp, int mode, bool quarters_ok, uint32_t v_widths, void* stream, uint32_t* sched) {
  StepArgs a;
  a.desc = d_desc;
  a.n_tensors = n;
  a.total_tiles = total;
  a.tables = ctx->d_tables;
  a.stats = d_stats;
  a.beta1 = hp->beta1;
  a.omb1 = 1.0f - hp->beta1;
  a.beta2 = hp->beta2;
  a.omb2 = 1.0f - hp->beta2;
  // reciprocal bias corrections 1/(1 - beta^t): double arithmetic, one rounding to fp32
  a.ibc1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(hp->beta1), static_cast<double>(hp->step))));
  a.ibc2 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(hp->beta2), static_cast<double>(hp->step))));
  a.eps = hp->eps;
  a.lr = hp->lr;
  a.decay = 1.0f - hp->lr * hp->weight_decay;
  a.lgK = static_cast<uint32_t>(lg_block(hp->block));
  a.v_widths = v_widths;

  // statistics: all of them, or only the gradient's (the flag for all wins)
  const int stats = (hp->flags & STQ_FLAG_STATS) ? 1 : ((hp->flags & STQ_FLAG_STATS_GRAD) ? 2 : 0);
  const bool want_stats = stats != 0;
  // every variant fits six waves per SIMD (three workgroups per CU) except the wide-state one (two)
  const uint32_t cap_cu = mode == 2 ? 2 : 8;
  const uint32_t per_cu = ctx->groups_per_cu < cap_cu ? ctx->groups_per_cu : cap_cu;
  const uint32_t wpg = kWavesPerGroup;
  const uint32_t max_groups = ctx->n_cu * per_cu;
  // Units of scheduling (see step_kernel): quarter tiles when whole tiles would leave waves idle and
  // every width keeps quarters word-aligned (multiples of 4 bits), else tiles.
  const bool quarters = quarters_ok && static_cast<uint64_t>(total) < static_cast<uint64_t>(max_groups) * wpg;
  a.quarter_units = quarters ? 1u : 0u;
  const uint64_t units = static_cast<uint64_t>(total) << (quarters ? 2 : 0);
  const uint64_t need_groups = (units + wpg - 1) / wpg;
  const uint32_t groups = static_cast<uint32_t>(need_groups < max_groups ? need_groups : max_groups);
  // order of the units under stripes (see step_kernel).  Without statistics interleaved chunks: pairs of units
  // once a wave has at least four (measured 2-3 % faster than single units between 5 and 11 units per wave:
  // a wave then owns whole cache lines of the scale arrays), four at a time from 24 on, single units in the
  // smallest launches so that every wave gets work.  With statistics few long chunks, because a wave flushes
  // its sums whenever its next unit lies in another tensor: one range per wave, or for the gradient's
  // statistics alone (a cheap flush) four units at a time in a large launch.
  const uint64_t n_waves = static_cast<uint64_t>(groups) * wpg;
  const uint64_t per_wave = (units + n_waves - 1) / n_waves;
  if (stats == 1) a.chunk = static_cast<uint32_t>(per_wave);
  else if (stats == 2) a.chunk = static_cast<uint32_t>(per_wave >= 64 ? 4 : per_wave);
  else a.chunk = per_wave >= 24 ? 4 : (per_wave >= 4 ? 2 : 1);
  if (ctx->chunk_override && !want_stats) a.chunk = ctx->chunk_override;
  // tickets (see step_kernel) for large launches; with statistics from a third of that size on, because the
  // stripes of those variants are few long chunks (measured: 61 K tiles 9 % faster with tickets, 42 K tiles 6 %
  // slower; without statistics 2 % faster and 12 % slower)
  const uint64_t min_units = want_stats ? ctx->ticket_min_units / 3 : ctx->ticket_min_units;
  a.sched = units < min_units ? nullptr : (sched ? sched : ctx->d_sched);
#ifdef STQ_TUNING_ENV
  if (std::getenv("STQ_NO_TICKETS")) a.sched = nullptr;
  if (std::getenv("STQ_TICKETS")) a.sched = sched ? sched : ctx->d_sched;
#endif
  return launch_step(a, hp->grad_dtype == 1, stats, mode, groups, stream) == 0 ? STQ_OK : STQ_EHIP;
}

}  // namespace stq

namespace {

// Stage n descriptors (already in pinned slot k, or copied there from `src`) into `dst` in stream order.
int upload_descs(stq_ctx* ctx, int k, const TensorDesc* src, size_t n, TensorDesc* dst, hipStream_t s) {
  if (src) std::memcpy(ctx->h_stage[k], src, sizeof(TensorDesc) * n);
  if (hipMemcpyAsync(dst, ctx->h_stage[k], sizeof(TensorDesc) * n, hipMemcpyHostToDevice, s) != hipSuccess) return STQ_EHIP;
  if (hipEventRecord(ctx->stage_done[k], s) != hipSuccess) return STQ_EHIP;
  return STQ_OK;
}

// The next pinned staging slot, free again (its upload of kRing calls ago has finished).
int next_stage_slot(stq_ctx* ctx, int* out) {
  const int k = ctx->ring_pos;
  if (int e = wait_slot_free(ctx->stage_done[k])) return e;
  ctx->ring_pos = (k + 1) % kRing;
  *out = k;
  return STQ_OK;
}

// Index of a device-resident tensor table that holds `descs`: one that already does (uploaded on this
// same stream, so the kernel is ordered after the upload), else the oldest, overwritten in stream order
// (after the kernels that read it).
int resident_table(stq_ctx* ctx, const std::vector<TensorDesc>& descs, hipStream_t s, int* out) {
  const size_t n = descs.size();
  int table = -1;
  for (int k = 0; k < kDescTables && table < 0; ++k)
    if (ctx->uploaded_on[k] == s && ctx->uploaded[k].size() == n &&
        std::memcmp(ctx->uploaded[k].data(), descs.data(), sizeof(TensorDesc) * n) == 0)
      table = k;
  if (table < 0) {
    table = ctx->desc_pos;
    int k = -1;
    if (int e = next_stage_slot(ctx, &k)) return e;
    ctx->uploaded[table].clear();  // whatever happens below, the old contents are no longer claimed
    if (int e = upload_descs(ctx, k, descs.data(), n, ctx->d_desc[table], s)) return e;
    ctx->desc_pos = (table + 1) % kDescTables;
    ctx->uploaded[table] = descs;
    ctx->uploaded_on[table] = s;
  }
  *out = table;
  return STQ_OK;
}

// Kernel variant for a set of descriptors: 0 in place, 1 widths change, 2 some state is (or becomes)
// 16 or 32 bits wide; and whether every width keeps quarter tiles word-aligned.
void classify(const TensorDesc* descs, uint32_t n, bool changes, int* mode, bool* quarters_ok, uint32_t* v_widths) {
  *mode = changes ? 1 : 0;
  *quarters_ok = true;
  *v_widths = 0;
  for (uint32_t l = 0; l < n; ++l) {
    const TensorDesc& d = descs[l];
    if (d.bv_out <= 8) *v_widths |= 1u << d.bv_out;
    if (is_wide(d.bm) || is_wide(d.bv) || is_wide(d.bm_out) || is_wide(d.bv_out)) *mode = 2;
    *quarters_ok = *quarters_ok && ((d.bm | d.bv | d.bm_out | d.bv_out) & 3u) == 0;
  }
}

// One launch of the step kernel.  new_plan/new_codes are null for the in-place step.
int step_impl(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, const stq_bits* plan,
              const stq_bits* new_plan, const stq_codes* new_codes, const stq_hparams* hp, void* stream) {
  if (int e = check_hparams(hp)) return e;
  if (!ctx) return STQ_EINVAL;
  std::vector<TensorDesc>& descs = ctx->descs;  // reserved at stq_init: no allocation per call
  uint32_t total = 0;
  if (int e = build_descs(ctx, tensors, n, plan, hp->block, true, descs, &total)) return e;
  if (new_plan) {
    for (uint32_t l = 0; l < n; ++l) {
      TensorDesc& d = descs[l];
      if (int e = check_bits_stored(new_plan[l].m_bits)) return e;
      if (int e = check_bits_stored(new_plan[l].v_bits)) return e;
      const uintptr_t span = static_cast<uintptr_t>(d.n_tiles) * 256;
      struct { uint32_t b_old, b_new; uint32_t* cur; void* dst; uint32_t** out; } st[2] = {
          {d.bm, new_plan[l].m_bits, d.m_codes, new_codes[l].m_codes, &d.m_out},
          {d.bv, new_plan[l].v_bits, d.v_codes, new_codes[l].v_codes, &d.v_out}};
      for (auto& x : st) {
        if (x.b_new == x.b_old && (x.dst == nullptr || x.dst == x.cur)) continue;  // stays in place
        // another width (or another buffer): the destination must be a distinct, aligned buffer
        if (!x.dst) return STQ_EINVAL;
        if (!aligned(x.dst, 256)) return STQ_EALIGN;
        const uintptr_t s0 = reinterpret_cast<uintptr_t>(x.cur), s1 = s0 + span * x.b_old;
        const uintptr_t d0 = reinterpret_cast<uintptr_t>(x.dst), d1 = d0 + span * x.b_new;
        if (s0 < d1 && d0 < s1) return STQ_EINVAL;
        *x.out = static_cast<uint32_t*>(x.dst);
      }
      d.bm_out = new_plan[l].m_bits;
      d.bv_out = new_plan[l].v_bits;
    }
  }
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);

  int table = -1;
  if (int e = resident_table(ctx, descs, s, &table)) return e;

  int mode;
  bool quarters_ok;
  uint32_t v_widths;
  classify(descs.data(), n, new_plan != nullptr, &mode, &quarters_ok, &v_widths);
  if (int e = launch_table(ctx, ctx->d_desc[table], n, total, ctx->d_stats, hp, mode, quarters_ok, v_widths, stream)) return e;
  if ((hp->flags & (STQ_FLAG_STATS | STQ_FLAG_STATS_GRAD)) != 0)
    for (uint32_t l = 0; l < n; ++l) ctx->stat_count[l] += tensors[l].numel;
  return STQ_OK;
}

}  // namespace

extern "C" {

int stq_step(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, const stq_bits* plan,
             const stq_hparams* hp, void* stream) {
  return step_impl(ctx, tensors, n, plan, nullptr, nullptr, hp, stream);
}

int stq_step_transition(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, const stq_bits* plan_old,
                        const stq_bits* plan_new, const stq_codes* new_codes, const stq_hparams* hp,
                        void* stream) {
  if (!plan_new || !new_codes) return STQ_EINVAL;
  return step_impl(ctx, tensors, n, plan_old, plan_new, new_codes, hp, stream);
}

int stq_step_static(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, const stq_bits* plan,
                    const stq_hparams* hp, void* stream) {
  if (int e = check_hparams(hp)) return e;
  if (!ctx || !tensors || !plan || n == 0) return STQ_EINVAL;
  if (n > kStaticMaxTensors) return STQ_ELIMIT;
  if (n > ctx->max_tensors) return STQ_EINVAL;
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // descriptors straight into a pinned staging slot, from there into this device's static table
  int k = -1;
  if (int e = next_stage_slot(ctx, &k)) return e;
  uint32_t total = 0;
  if (int e = fill_descs(ctx, tensors, n, plan, hp->block, true, ctx->h_stage[k], &total)) return e;
  int mode;
  bool quarters_ok;
  uint32_t v_widths;
  classify(ctx->h_stage[k], n, false, &mode, &quarters_ok, &v_widths);
  TensorDesc* table = static_cast<TensorDesc*>(ctx->static_scratch);
  uint32_t* sched = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(ctx->static_scratch) + kStaticTableBytes);
  if (int e = upload_descs(ctx, k, nullptr, n, table, s)) return e;
  // the scheduling words must be zero when the kernel starts: a kernel leaves them so, but the array is shared
  // by every caller on this GPU and may hold what an aborted launch left
  if (launch_fill_zero(sched, kSchedWords, stream) != 0) return STQ_EHIP;
  if (int e = launch_table(ctx, table, n, total, ctx->d_stats, hp, mode, quarters_ok, v_widths, stream, sched)) return e;
  if ((hp->flags & (STQ_FLAG_STATS | STQ_FLAG_STATS_GRAD)) != 0)
    for (uint32_t l = 0; l < n; ++l) ctx->stat_count[l] += tensors[l].numel;
  return STQ_OK;
}

int stq_grad_stats(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, uint32_t block, uint32_t grad_dtype,
                   void* stream) {
  if (grad_dtype > 1) return STQ_EINVAL;
  if (!ctx || !tensors || n == 0 || n > ctx->max_tensors) return STQ_EINVAL;
  std::vector<stq_bits> any(n, stq_bits{8, 8});  // the widths play no part here
  std::vector<TensorDesc> descs;
  uint32_t total = 0;
  if (int e = build_descs(ctx, tensors, n, any.data(), block, true, descs, &total)) return e;
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  int table = -1;
  if (int e = resident_table(ctx, descs, static_cast<hipStream_t>(stream), &table)) return e;
  if (launch_grad_stats(ctx->d_desc[table], n, total, ctx->d_stats, grad_dtype == 1, grad_stats_groups(ctx->n_cu, total), stream) != 0)
    return STQ_EHIP;
  for (uint32_t l = 0; l < n; ++l) ctx->stat_count[l] += tensors[l].numel;
  return STQ_OK;
}

int stq_stats(stq_ctx* ctx, stq_layer_stats* out, uint32_t n, void* stream) {
  if (!ctx || !out || n == 0 || n > ctx->max_tensors) return STQ_EINVAL;
  for (uint32_t l = 0; l < n; ++l) if (ctx->stat_count[l] == 0) return STQ_ESTATE;
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t bytes = sizeof(double) * kStatSlots * n;
  if (hipMemcpyAsync(ctx->h_stats, ctx->d_stats, bytes, hipMemcpyDeviceToHost, s) != hipSuccess) return STQ_EHIP;
  if (launch_fill_zero(reinterpret_cast<uint32_t*>(ctx->d_stats), bytes / 4, stream) != 0) return STQ_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return STQ_EHIP;
  for (uint32_t l = 0; l < n; ++l) {
    const double* a = ctx->h_stats + static_cast<size_t>(l) * kStatSlots;
    stq_layer_stats& o = out[l];
    o.count = ctx->stat_count[l];
    o.g_sum = a[kGSum]; o.g_abs_sum = a[kGAbsSum]; o.g_sq_sum = a[kGSqSum];
    o.m_sum = a[kMSum]; o.m_sq_sum = a[kMSqSum]; o.m_err_sq = a[kMErrSq];
    o.v_sum = a[kVSum]; o.v_sq_sum = a[kVSqSum]; o.v_err_sq = a[kVErrSq];
    uint32_t mx[4];
    std::memcpy(mx, &a[kMaxGM], 16);
    std::memcpy(&o.g_absmax, &mx[0], 4);
    std::memcpy(&o.m_absmax, &mx[1], 4);
    std::memcpy(&o.v_absmax, &mx[2], 4);
    ctx->stat_count[l] = 0;
  }
  return STQ_OK;
}

int stq_repack(stq_ctx* ctx, uint64_t numel, uint32_t block, int state, const void* src,
               uint32_t src_bits, void* dst, uint32_t dst_bits, void* stream) {
  // one job of stq_repack_many: the same checks, the same kernel
  if (state != 0 && state != 1) return STQ_EINVAL;
  stq_repack_job j;
  j.numel = numel;
  j.src_codes = src;
  j.dst_codes = dst;
  j.state = static_cast<uint8_t>(state);
  j.src_bits = static_cast<uint8_t>(src_bits <= 255 ? src_bits : 255);
  j.dst_bits = static_cast<uint8_t>(dst_bits <= 255 ? dst_bits : 255);
  return stq_repack_many(ctx, &j, 1, block, stream);
}

int stq_repack_many(stq_ctx* ctx, const stq_repack_job* jobs, uint32_t n, uint32_t block, void* stream) {
  if (!ctx || !jobs || n == 0 || n > 2 * ctx->max_tensors) return STQ_EINVAL;
  if (lg_block(block) < 0) return STQ_EBLOCK;
  std::vector<RepackJob> table(n);
  uint64_t total = 0;
  for (uint32_t i = 0; i < n; ++i) {
    const stq_repack_job& j = jobs[i];
    if (!j.src_codes || !j.dst_codes || j.numel == 0 || j.state > 1) return STQ_EINVAL;
    if (int e = check_bits(j.src_bits)) return e;
    if (int e = check_bits(j.dst_bits)) return e;
    if (!aligned(j.src_codes, 256) || !aligned(j.dst_codes, 256)) return STQ_EALIGN;
    const uint64_t tiles = (j.numel + kTile - 1) / kTile;
    if (total + tiles > 0xFFFFFFFFull) return STQ_EINVAL;
    const uintptr_t s0 = reinterpret_cast<uintptr_t>(j.src_codes), s1 = s0 + tiles * 256 * j.src_bits;
    const uintptr_t d0 = reinterpret_cast<uintptr_t>(j.dst_codes), d1 = d0 + tiles * 256 * j.dst_bits;
    if (s0 < d1 && d0 < s1) return STQ_EINVAL;
    RepackJob& r = table[i];
    r.src = static_cast<const uint32_t*>(j.src_codes);
    r.dst = static_cast<uint32_t*>(j.dst_codes);
    r.numel = j.numel;
    r.tile_begin = static_cast<uint32_t>(total);
    r.n_tiles = static_cast<uint32_t>(tiles);
    r.b_old = j.src_bits;
    r.b_new = j.dst_bits;
    r.lut = repack_lut_index(j.state, j.src_bits, j.dst_bits);
    r.pad = 0;
    total += tiles;
  }
  DeviceGuard g(ctx->device);
  if (!g.ok) return STQ_EHIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int k = ctx->jobs_pos;
  ctx->jobs_pos = (k + 1) % kRing;
  if (int e = wait_slot_free(ctx->jobs_done[k])) return e;
  std::memcpy(ctx->h_jobs[k], table.data(), sizeof(RepackJob) * n);
  if (hipMemcpyAsync(ctx->d_jobs, ctx->h_jobs[k], sizeof(RepackJob) * n, hipMemcpyHostToDevice, s) != hipSuccess)
    return STQ_EHIP;
  if (hipEventRecord(ctx->jobs_done[k], s) != hipSuccess) return STQ_EHIP;
  RepackManyArgs a;
  a.jobs = ctx->d_jobs;
  a.n_jobs = n;
  a.total_tiles = static_cast<uint32_t>(total);
  a.luts = ctx->d_luts;
  // one wave per workgroup, chunks of kRepackChunk tiles; at most eight waves per SIMD resident
  const uint64_t need = (total + kRepackChunk - 1) / kRepackChunk;
  const uint64_t cap = static_cast<uint64_t>(ctx->n_cu) * 32;
  return launch_repack_many(a, static_cast<uint32_t>(need < cap ? need : cap), stream) == 0 ? STQ_OK : STQ_EHIP;
}

}  // extern "C"
