// Structures shared by the host API and the gfx950 kernels of this library.
#pragma once
#include <cstdint>

namespace stq {

constexpr int kTile = 2048;         // elements per tile = 64 lanes x 32 codes
constexpr uint32_t kRepackChunk = 8;  // consecutive tiles a wave of repack_many_kernel converts at a time (1..16 measured alike)
constexpr int kWavesPerGroup = 8;   // 512-thread workgroups
constexpr int kStatSlots = 16;      // 8-byte accumulator slots per tensor
constexpr uint32_t kSchedWords = 2;  // the ticket counter of a launch and the count of workgroups that have left

// Device-resident description of one tensor for the step kernel.
struct TensorDesc {
  float* param;
  const void* grad;
  uint32_t* m_codes;
  float* m_scales;
  uint32_t* v_codes;
  float* v_scales;
  uint64_t numel;
  uint32_t tile_begin;  // index of this tensor's first tile in the launch-wide tile order
  uint32_t n_tiles;
  uint32_t bm, bv;      // widths of the stored codes
  uint32_t* m_out;      // where the new codes go: the same buffers, or others when a width changes
  uint32_t* v_out;
  uint32_t bm_out, bv_out;
};

// Accumulator slots (doubles unless noted).
enum StatSlot {
  kGSum = 0, kGAbsSum, kGSqSum, kMSum, kMSqSum, kMErrSq, kVSum, kVSqSum, kVErrSq,
  kMaxGM,   // two uint32: bit patterns of max|g| (low word) and max|m| (high word)
  kMaxV     // low uint32: bit pattern of max v
};

struct StepArgs {
  const TensorDesc* desc;
  uint32_t n_tensors;
  uint32_t total_tiles;
  const uint32_t* tables;  // kTabWords words, see stq_tables.h
  double* stats;           // [n_tensors][kStatSlots]
  float beta1, omb1, beta2, omb2;
  float ibc1, ibc2;        // reciprocal bias corrections 1/(1-beta^t)
  float eps, lr, decay;    // decay = 1 - lr*weight_decay
  uint32_t lgK;            // log2 of the block size: 6, 7 or 8
  uint32_t chunk;          // consecutive units a wave takes at a time, see step_kernel
  uint32_t quarter_units;  // 1: a unit is a quarter tile (small launches whose widths keep quarters word-aligned)
  uint32_t v_widths;       // bit b set: some second moment may be quantized at width b in this launch
  uint32_t* sched;         // kSchedWords words, zero between launches: the ticket counters and the count of
                           // workgroups that have left; null: no tickets, every wave walks its own stripes
                           // (see step_kernel)
};

struct ZeroArgs {
  uint32_t* m_codes; float* m_scales; uint32_t* v_codes; float* v_scales;
  uint64_t numel;
  uint32_t n_tiles, bm, bv, scales_per_tile;
};

// One width change inside a batched re-pack launch.
struct RepackJob {
  const uint32_t* src; uint32_t* dst;
  uint64_t numel;
  uint32_t tile_begin, n_tiles;  // position in the launch-wide tile order
  uint32_t b_old, b_new;
  uint32_t lut;                  // index of the conversion table, see repack_lut_index
  uint32_t pad;
};
constexpr uint32_t kRepackLuts = 2 * 7 * 7;  // (state, old width, new width)
constexpr uint32_t repack_lut_index(uint32_t state, uint32_t b_old, uint32_t b_new) {
  return (state * 7 + (b_old - 2)) * 7 + (b_new - 2);
}
struct RepackManyArgs {
  const RepackJob* jobs;
  uint32_t n_jobs, total_tiles;
  const uint32_t* luts;  // [kRepackLuts][256] words
};

// Launchers implemented in stq_step.hip and stq_kernels.hip.  `stream` is a hipStream_t.  Return a hipError_t as int.
// stats: 0 none, 1 every statistic, 2 the gradient's only.
int launch_step(const StepArgs& a, bool grad_bf16, int stats, int mode, uint32_t groups, void* stream);
int launch_zero(const ZeroArgs& a, void* stream);
int launch_repack_many(const RepackManyArgs& a, uint32_t groups, void* stream);
int launch_grad_stats(const TensorDesc* desc, uint32_t n_tensors, uint32_t total_tiles, double* stats, bool grad_bf16,
                      uint32_t groups, void* stream);
int launch_fill_zero(uint32_t* p, uint64_t words, void* stream);

}  // namespace stq
