// Host-side internals shared by the sources that implement the C ABI: the context, argument
// checks, and the one place that configures and launches the step kernel over a device-resident
// tensor table.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "stq.h"
#include "stq_device.h"

namespace stq {

constexpr int kRing = 16;       // pinned staging slots for descriptor uploads
constexpr uint64_t kTicketMinUnits = 160000;  // launches of at least this many units draw tickets (see step_kernel):
                                              // about 0.3 G elements; below, the barrier costs more than the order gains
constexpr int kDescTables = 4;  // device-resident tensor tables kept: a caller that alternates between a
                                // few argument sets (two gradient buffers, say) uploads each only once

}  // namespace stq

struct stq_ctx {
  int device = -1;
  uint32_t max_tensors = 0;
  uint32_t n_cu = 0;
  uint32_t groups_per_cu = 3;    // resident workgroups per CU the plain step kernel is launched for
  uint32_t chunk_override = 0;  // tuning aid: STQ_CHUNK in the environment
  uint64_t ticket_min_units = stq::kTicketMinUnits;  // see stq_set_schedule
  uint32_t* d_tables = nullptr;
  stq::TensorDesc* d_desc[stq::kDescTables] = {nullptr, nullptr, nullptr, nullptr};
  double* d_stats = nullptr;
  uint32_t* d_sched = nullptr;   // ticket counter and leave count of the step kernel (zero between launches)
  stq::TensorDesc* h_stage[stq::kRing] = {};  // pinned
  hipEvent_t stage_done[stq::kRing] = {};
  int ring_pos = 0;
  uint32_t* d_luts = nullptr;                // every conversion table of the re-pack, kRepackLuts x 256 words
  stq::RepackJob* d_jobs = nullptr;          // 2 * max_tensors
  stq::RepackJob* h_jobs[stq::kRing] = {};  // pinned
  hipEvent_t jobs_done[stq::kRing] = {};
  int jobs_pos = 0;
  double* h_stats = nullptr;                 // pinned, max_tensors * kStatSlots
  std::vector<stq::TensorDesc> uploaded[stq::kDescTables];  // what each d_desc currently holds
  hipStream_t uploaded_on[stq::kDescTables] = {nullptr, nullptr, nullptr, nullptr};  // the stream that uploaded it
  std::vector<stq::TensorDesc> descs;        // descriptors of the call in progress (capacity max_tensors)
  void* static_scratch = nullptr;            // this device's static table of stq_step_static
  int desc_pos = 0;                          // next table to replace
  std::vector<uint64_t> stat_count;          // elements accumulated per tensor since the last stq_stats
};

namespace stq {

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int check_bits(uint32_t b) { return (b >= 2 && b <= 8) ? STQ_OK : STQ_EBITS; }
inline bool is_wide(uint32_t b) { return b == 16 || b == 32; }
// widths a state can be stored at: the quantized ones, and 16 (bfloat16) and 32 (fp32) as they are
inline int check_bits_stored(uint32_t b) { return (is_wide(b) || check_bits(b) == STQ_OK) ? STQ_OK : STQ_EBITS; }

inline int lg_block(uint32_t K) {
  switch (K) { case 64: return 6; case 128: return 7; case 256: return 8; default: return -1; }
}

// A pinned staging slot may be written again once the upload it last fed has finished.  Asking is cheap and
// almost always enough (the ring is long); waiting is the rare fallback -- on this runtime a wait on an event
// can take as long as the work queued behind it.
inline int wait_slot_free(hipEvent_t done) {
  const hipError_t q = hipEventQuery(done);
  if (q == hipSuccess) return STQ_OK;
  if (q != hipErrorNotReady) { (void)hipGetLastError(); return STQ_EHIP; }
  (void)hipGetLastError();
  return hipEventSynchronize(done) == hipSuccess ? STQ_OK : STQ_EHIP;
}

struct DeviceGuard {  // makes the context's device current for the duration of a call
  int prev = -1; bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    if (prev == dev) prev = -1;
  }
  ~DeviceGuard() { if (ok && prev >= 0) (void)hipSetDevice(prev); }
};

// Checks the hyper-parameters of a step (Adam's own preconditions).
int check_hparams(const stq_hparams* hp);

// Fills the descriptors of n tensors at the widths of `plan` (new codes in place) and the launch-wide tile count.
int fill_descs(const stq_ctx* ctx, const stq_tensor* t, uint32_t n, const stq_bits* plan, uint32_t K,
               bool need_param_grad, TensorDesc* out, uint32_t* total_tiles);
int build_descs(const stq_ctx* ctx, const stq_tensor* t, uint32_t n, const stq_bits* plan, uint32_t K,
                bool need_param_grad, std::vector<TensorDesc>& out, uint32_t* total_tiles);

// Launches the step kernel over the device-resident table `d_desc` of n tensors / total_tiles tiles.
// mode: 0 in place, 1 widths change, 2 some state is (or may become) 16 or 32 bits wide.
// quarters_ok: every width of the launch is a multiple of 4 bits.
// v_widths: bit b set if a second moment may be quantized at width b in this launch (the kernel loads the search
// tables of these widths only).  sched: the two scheduling words the launch uses (null: the context's own).
int launch_table(stq_ctx* ctx, const TensorDesc* d_desc, uint32_t n, uint32_t total_tiles, double* d_stats,
                 const stq_hparams* hp, int mode, bool quarters_ok, uint32_t v_widths, void* stream,
                 uint32_t* sched = nullptr);

// Workgroups (of four waves) for the gradient-statistics kernel: at most eight per CU, at least one tile per wave.
inline uint32_t grad_stats_groups(uint32_t n_cu, uint32_t total_tiles) {
  const uint64_t need = (static_cast<uint64_t>(total_tiles) + 3) / 4, cap = static_cast<uint64_t>(n_cu) * 8;
  return static_cast<uint32_t>(need < cap ? need : cap);
}

}  // namespace stq
