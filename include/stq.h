/*
 * stq.h -- C ABI of the MI355X (gfx950) quantized Adam step of STQuant.
 *
 * The library implements the per-layer loop body of the paper's Algorithm 1
 * (moment update, block-wise Quantize of m [linear symmetric] and v
 * [logarithmic] per Section 3.5, bias correction of the quantized moments,
 * decoupled-weight-decay update), the per-layer statistics the Score Engine of
 * Section 3.3 consumes, the conversion of stored codes when Map (Section 3.4)
 * changes a layer's bit-width, the host-side decision itself, and the same loop
 * with the decision and the bit plan resident on the device (stq_engine_*).
 *
 * Conventions
 *   - Every function returns STQ_OK (0) or a negative STQ_E* code.  Nothing
 *     throws, aborts or prints.  stq_strerror() names a code.
 *   - "device" pointers are HIP device memory on the context's GPU, owned by the
 *     caller; only stq_init and stq_engine_create allocate, only stq_destroy and
 *     stq_engine_destroy free.  "host" pointers are ordinary process memory.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     stq_zero_state, stq_step, stq_step_transition, stq_repack and stq_repack_many
 *     are asynchronous on that stream; stq_stats synchronises it.  stq_step,
 *     stq_step_transition and stq_grad_stats keep the tensor tables of the last four
 *     distinct argument sets on the device: a call whose tensors, plan and block size
 *     equal one of those, on the same stream, is one kernel launch and nothing else
 *     (no upload, no wait, no allocation).  Any other call, and every stq_repack and
 *     stq_repack_many, first uploads a small table from pinned host memory (sixteen staging slots
 *     in turn; a slot whose last upload has not finished yet is waited for); such a
 *     call cannot be recorded into a HIP graph.  (The step number reaches the kernel as launch arguments, so a
 *     recorded launch repeats its own step.)  stq_engine_step is asynchronous too; with
 *     grads = NULL it consists of kernel launches only.
 *   - One context serves one stream at a time.  Calls on one context must not
 *     overlap from several host threads.  A context may move to another stream after
 *     the caller has ordered the new stream behind the old one's work; tensor tables
 *     are then uploaded again on the new stream.
 *   - Gradients, parameters and hyper-parameters must be finite.  A non-finite
 *     gradient makes the codes of its tile meaningless (only the tensors' own
 *     buffers are written; no address depends on data).  It shows in the statistics:
 *     g_sq_sum of that tensor is then not finite (Inf or NaN; also for a finite
 *     gradient whose square overflows fp32), so a loss-scaling caller can run
 *     stq_grad_stats + stq_stats first and skip the step.
 *
 * Storage of one state (m or v) of a tensor of `numel` elements, block K, width b:
 *   codes : tiles of 2048 elements, 64*b 32-bit words per tile.  Inside a tile,
 *           "lane" j (0..63) owns elements tile*2048 + 256*i + 4*j + e (i=0..7,
 *           e=0..3) and writes their codes in the order n = 4*i+e, LSB first,
 *           into a stream of 32*b bits; word p of that stream is stored at word
 *           index tile*64*b + p*64 + j.  Pad elements (>= numel) have code bits 0.
 *   scales: fp32, one per block of K consecutive elements, zero-padded to
 *           2048/K entries per tile.
 *   stq_state_bytes() returns both sizes.  Both arrays must be 256-byte aligned.
 *   Values: first moment  m = scale * (u - qmax)/qmax,  qmax = 2^(b-1)-1, u = code;
 *           second moment v = scale * 2^(-(2^b-1-c) * 2^(4-b)),  c = code.
 *   Widths 16 and 32 (see stq_bits) use the same tile format with 16- or 32-bit codes and
 *   no scales (the scale arrays must still be passed; they are left untouched).
 */
#ifndef STQ_H
#define STQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STQ_OK = 0,
  STQ_EINVAL = -1,  /* null pointer, zero size, count above the context's limit */
  STQ_EALIGN = -2,  /* a device buffer is not aligned as required */
  STQ_EBITS = -3,   /* a width outside 2..8 (and, where a stored state is meant, other than 16 or 32) */
  STQ_EBLOCK = -4,  /* block size not 64, 128 or 256 */
  STQ_EDEVICE = -5, /* no such device, or not a gfx950 GPU */
  STQ_EHIP = -6,    /* a HIP runtime call failed */
  STQ_ESTATE = -7,  /* stq_stats called with nothing accumulated for that many tensors */
  STQ_ELIMIT = -8   /* stq_step_static: more tensors than its static table holds */
};

typedef struct stq_ctx stq_ctx; /* opaque, owned by the library */

/* One parameter tensor = one "layer" l of Algorithm 1. */
typedef struct {
  void* param;        /* device, fp32[numel], 16-byte aligned, updated in place            */
  const void* grad;   /* device, fp32[numel] or bf16[numel] (hparams.grad_dtype), 16-byte aligned */
  uint64_t numel;     /* N_l >= 1                                                           */
  void* m_codes;      /* device, first-moment codes, size from stq_state_bytes, in place    */
  float* m_scales;    /* device, first-moment block scales, in place                        */
  void* v_codes;      /* device, second-moment codes                                        */
  float* v_scales;    /* device, second-moment block scales                                 */
} stq_tensor;

/* bit_plan[l]: the widths b_{l,t} of layer l's two states: 2..8 (block-quantized codes), or 16 / 32,
 * the wide members of the paper's width set {4, 8, 16, 32}: the state is then kept without scales as
 * the bfloat16 rounding (16) or the fp32 value itself (32) of each element, in the same tile format
 * with 16- or 32-bit codes (the upper half of the fp32 bit pattern, or all of it).  stq_repack and
 * stq_repack_many convert between the quantized widths only; a change from or to a wide format
 * goes through stq_step_transition. */
typedef struct { uint8_t m_bits, v_bits; } stq_bits;

/* Inputs of Algorithm 1 that the step needs. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay; /* eta >= 0, 0 <= beta1, beta2 < 1, epsilon > 0, lambda; all
                                                finite, else STQ_EINVAL                      */
  uint32_t step;       /* t >= 1, used for the bias corrections 1 - beta^t                */
  uint32_t block;      /* block size K: 64, 128 or 256                                    */
  uint32_t grad_dtype; /* 0 = fp32, 1 = bf16                                              */
  uint32_t flags;      /* STQ_FLAG_* below                                                */
} stq_hparams;
#define STQ_FLAG_STATS 1u      /* accumulate every per-layer statistic of stq_layer_stats during this step */
#define STQ_FLAG_STATS_GRAD 2u /* accumulate only the gradient's (count, g_sum, g_abs_sum, g_sq_sum, g_absmax:
                                  all that stq_decide reads); the moments' fields stay 0.  Cheaper (about 2 % of a
                                  step against 10 %).  STQ_FLAG_STATS wins if both are set. */

/* Host copy of one layer's accumulated statistics (Section 3.3 inputs plus the
 * moments' own statistics and quantization error).  m and v are the new moments
 * BEFORE quantization; *_err_sq is the sum of (x - Quantized(x))^2. */
typedef struct {
  uint64_t count;
  double g_sum, g_abs_sum, g_sq_sum; float g_absmax;
  double m_sum, m_sq_sum, m_err_sq;  float m_absmax;
  double v_sum, v_sq_sum, v_err_sq;  float v_absmax;
} stq_layer_stats;

/* The O(1) state of the decision: the three global EMAs of Eq. 4 / Section 3.3.3. */
typedef struct { double n_ema, r_ema, v_ema; } stq_decide_state;

/* Parameters of the decision.  The paper's values: phi = 7.2, thr = {6.8, 12, 24},
 * bits = {4, 8, 16, 32}; alpha, tau and eps are not given there.  Only widths
 * 2..8 can be stored by this library; stq_decide itself maps to whatever `bits`
 * holds.  `bits` has n_thr+1 entries: width = bits[#{i : thr[i] <= score}].  The
 * second-moment width is mapped from score + v_offset. */
typedef struct {
  double alpha, tau, phi, eps, v_offset;
  uint32_t flags;  /* bit 0: r_l = sigma(g)/(E|g|+eps) as in Algorithm 1 instead of Eq. 3's CV of |g|;
                      bits 1..3: the ablations of the paper's component study, see below */
  uint32_t n_thr;
  const double* thr;   /* host, ascending */
  const uint8_t* bits; /* host */
} stq_decide_cfg;
#define STQ_DECIDE_R_ALG1 1u
#define STQ_DECIDE_NO_DUAL 2u     /* score without the intensity and variation terms ("w/o Dual Factor") */
#define STQ_DECIDE_NO_TEMPORAL 4u /* score without log2 S_t ("w/o Temporal Factor") */
#define STQ_DECIDE_NO_SPATIAL 8u  /* score without log2(v_l / v_global) ("w/o Spatial Factor") */

/* Create a context on HIP device `device` (must be gfx950) for up to
 * max_tensors tensors per call.  Builds the level/threshold tables of the two
 * quantizers and allocates the descriptor and statistics buffers. */
int stq_init(stq_ctx** out, int device, uint32_t max_tensors);

/* Order in which the step kernel takes the tiles of a launch (results do not depend on it, only speed; the
 * statistics' sums differ in the last bits as with any other order of addition).  Launches of at least
 * `ticket_min_tiles` tiles (quarter tiles in very small launches) use the ticket schedule: workgroups draw
 * runs of neighbouring tiles from a counter in device memory and their waves work on them in step, so the
 * chip sweeps every array front to back inside one compact window -- worth 10-15 % of bandwidth on
 * multi-gigabyte workloads, a loss on small ones, where each wave keeps walking its own stripes.
 * Steps that gather statistics switch at a third of the value.  0 restores the default (about 0.3 G
 * elements); UINT64_MAX never uses tickets.  Host only. */
int stq_set_schedule(stq_ctx* ctx, uint64_t ticket_min_tiles);

/* Synchronise the device and free everything the context owns. */
int stq_destroy(stq_ctx* ctx);

/* Sizes in bytes of the code and scale arrays of one state (see "Storage"). Host only. */
int stq_state_bytes(uint64_t numel, uint32_t block, uint32_t bits,
                    uint64_t* code_bytes, uint64_t* scale_bytes);

/* Write Algorithm 1's initial state m_0 = v_0 = 0 into the n tensors' code and
 * scale arrays at the widths of bit_plan (param and grad are not touched and
 * may be NULL). */
int stq_zero_state(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n,
                   const stq_bits* bit_plan, uint32_t block, void* hip_stream);

/* One quantized Adam step over n tensors (Algorithm 1, the "for each layer"
 * body, with the stored states as m_{t-1}, v_{t-1}): params, codes and scales
 * are updated in place; with STQ_FLAG_STATS the statistics of tensor l are
 * added to accumulator l.  tensors and bit_plan are host arrays of n entries,
 * read before the call returns.  One kernel launch, no host synchronisation. */
int stq_step(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n,
             const stq_bits* bit_plan, const stq_hparams* hp, void* hip_stream);

/* stq_step for callers that cannot allocate device memory or wait for an allocator (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step, the
 * same kernel and the same results, but the kernel's scratch memory -- the tensor table it reads
 * and the scheduling words of large launches -- lives in a static device array of the library
 * (STQ_STATIC_MAX_TENSORS entries of 96 bytes + 256 bytes, about 96 KiB per GPU, held until the
 * process ends) instead of the context's buffers.  The call allocates nothing on host or device:
 * it fills a pinned staging slot of the context, copies it to the static table in stream order,
 * clears the scheduling words with a small kernel and launches.  n above STQ_STATIC_MAX_TENSORS gives STQ_ELIMIT
 * (n above the context's max_tensors STQ_EINVAL).  Every call on a GPU, from any context, uses
 * that GPU's one table: calls that overlap on one GPU (two streams, two contexts) race; on one
 * stream they are ordered.  Statistics flags work as in stq_step (the context's accumulators). */
#define STQ_STATIC_MAX_TENSORS 1024u
int stq_step_static(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n,
                    const stq_bits* bit_plan, const stq_hparams* hp, void* hip_stream);

/* Destination of one tensor's new codes in stq_step_transition. */
typedef struct {
  void* m_codes; /* device, 256-byte aligned, sized by stq_state_bytes at the NEW width; may be NULL
                    or the tensor's own m_codes when that width does not change */
  void* v_codes;
} stq_codes;

/* The step in which Map's new plan takes effect, as Algorithm 1 is written: the
 * layer's new width b_{l,t} is set before the layer loop, so the stored states
 * m_{t-1}, v_{t-1} are read at the widths of plan_old (from tensors[l].m_codes /
 * v_codes) and the new states are quantized and stored at the widths of plan_new,
 * into new_codes[l] (scales stay in the tensor's scale arrays; a state whose width
 * does not change may stay in place).  No separate conversion pass and no extra
 * rounding of the old state.  A changed state's destination must not overlap its
 * source.  Otherwise as stq_step; afterwards the caller uses plan_new and the new
 * buffers. */
int stq_step_transition(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n,
                        const stq_bits* plan_old, const stq_bits* plan_new,
                        const stq_codes* new_codes, const stq_hparams* hp, void* hip_stream);

/* Add the statistics of the gradients alone (count, g_sum, g_abs_sum, g_sq_sum, g_absmax) of the n
 * tensors to accumulators 0..n-1, without a step: for a caller that follows Algorithm 1's written order
 * (statistics of g_t -> stq_stats -> stq_decide -> stq_step_transition of the same step t).  One pass
 * over the gradients; only tensors[l].grad and numel are read (the other fields must still be valid).
 * Asynchronous; uploads a small table like stq_step. */
int stq_grad_stats(stq_ctx* ctx, const stq_tensor* tensors, uint32_t n, uint32_t block,
                   uint32_t grad_dtype, void* hip_stream);

/* Copy accumulators 0..n-1 to `out` (host, n entries), synchronise, and clear
 * them on the device.  Sums are order-dependent in the last bits; the maxima
 * are exact. */
int stq_stats(stq_ctx* ctx, stq_layer_stats* out, uint32_t n, void* hip_stream);

/* Convert the codes of one state of one tensor from src_bits to dst_bits after
 * Map changed the layer's width.  state: 0 = first moment, 1 = second moment.
 * Code-domain conversion: the new code is the one the dst_bits quantizer gives
 * the old code's value in a block of scale 1; the scales array is shared by
 * both widths and is not touched.  src and dst must not overlap.  The same as
 * stq_repack_many with one job. */
int stq_repack(stq_ctx* ctx, uint64_t numel, uint32_t block, int state,
               const void* src_codes, uint32_t src_bits,
               void* dst_codes, uint32_t dst_bits, void* hip_stream);

/* One width change of one state, for stq_repack_many: the arguments of stq_repack. */
typedef struct {
  uint64_t numel;
  const void* src_codes; /* device, 256-byte aligned */
  void* dst_codes;       /* device, 256-byte aligned, must not overlap src_codes */
  uint8_t state;         /* 0 = first moment, 1 = second moment */
  uint8_t src_bits, dst_bits;
} stq_repack_job;

/* n width changes (as stq_repack, one per job) in ONE kernel launch: what Map's new
 * plan asks for after a decision, when many layers change at once.  jobs is a host
 * array, read before the call returns; n may not exceed twice the context's
 * max_tensors.  Jobs must not overlap each other's destinations. */
int stq_repack_many(stq_ctx* ctx, const stq_repack_job* jobs, uint32_t n, uint32_t block,
                    void* hip_stream);

/* Host-side bit-width decision for n layers (Algorithm 1, the "if t mod U = 0
 * or t < 5" body; Eq. 2, 3, 4, 7, 8; Section 3.4 score and Map): updates *ema and
 * writes plan_out[l].  score_out (host, n doubles) may be NULL.  Linear in n. */
int stq_decide(stq_decide_state* ema, const stq_layer_stats* stats, uint32_t n,
               const stq_decide_cfg* cfg, uint32_t step, stq_bits* plan_out,
               double* score_out);

/* Algorithm 1's update cadence: 1 when the decision runs at step t (t mod U = 0, or t < 5), else 0.
 * U = 0 means "only during the first steps". */
int stq_decide_due(uint32_t step, uint32_t update_every);

/* ---- Device-resident precision loop -------------------------------------------------
 * Algorithm 1's whole iteration (the layer loop, and every U steps the statistics ->
 * EMAs -> score -> Map body) with the bit plan, the EMAs and the tensor table living
 * on the device: stq_engine_step only enqueues kernels, nothing is copied back and the
 * host never waits.  The decision is the one stq_decide takes (same formulas, fp64,
 * same order of the sums over the layers; log2 is the device library's).  Two orders:
 *   default: the statistics of g_t are a by-product of step t's kernel (no extra pass)
 *     and the decision takes effect in step t+1, which reads each state at its old
 *     width and writes it at the new one (the width-changing step of stq_step_transition);
 *   STQ_ENGINE_ALG1_ORDER: as Algorithm 1 is written -- on a decision step a pass over
 *     the gradients gathers the statistics, Map sets the widths, and the layer loop of
 *     the SAME step t writes the states at the new widths (one more read of the
 *     gradients on decision steps). */
typedef struct stq_engine stq_engine;
#define STQ_ENGINE_ALG1_ORDER 1u

/* tensors[l] (host array of n): the parameter, gradient, scale arrays and FIRST code
 * buffers, holding states at the widths of initial_plan (stq_zero_state, or a restored
 * checkpoint); second[l]: a SECOND code buffer per state.  Every code buffer must hold
 * the state at capacity_bits (stq_state_bytes), and capacity_bits must be at least every
 * width of initial_plan and of cfg->bits; scale arrays are needed even while a state is
 * 16 or 32 bits wide.  A state lives in one of its two buffers and moves to the other
 * when its width changes.  cfg->n_thr may not exceed 15; cfg is copied.  The EMAs start
 * at *ema (zeros if NULL).  flags: 0 or STQ_ENGINE_ALG1_ORDER.  The engine keeps the
 * context's device; destroy it before the context. */
int stq_engine_create(stq_ctx* ctx, stq_engine** out, const stq_tensor* tensors,
                      const stq_codes* second, uint32_t n, const stq_bits* initial_plan,
                      uint32_t capacity_bits, uint32_t block, const stq_decide_cfg* cfg,
                      const stq_decide_state* ema, uint32_t flags, void* hip_stream);

/* Step hp->step of the loop (hp->block must be the engine's; STQ_FLAG_STATS in hp->flags
 * is ignored: the engine collects statistics exactly when stq_decide_due(hp->step,
 * update_every) says so, and then runs the decision kernel after the step).  grads: NULL,
 * or a host array of n device pointers that replace the tensors' gradient buffers from
 * this step on (read before the call returns).  Steps must be enqueued in order on one
 * stream. */
int stq_engine_step(stq_engine* e, const stq_hparams* hp, uint32_t update_every,
                    const void* const* grads, void* hip_stream);

/* Carry a waiting decision over a checkpoint (default order only): next[l] (host array of n) are the widths
 * the engine's first step shall write, i.e. the next[] that stq_engine_read returned when the checkpoint was
 * taken; the states are still stored at the widths given to stq_engine_create.  Call it between
 * stq_engine_create and the first stq_engine_step (later, or in STQ_ENGINE_ALG1_ORDER: STQ_ESTATE).  Every
 * width must be one of the engine's ladder (cfg->bits), else STQ_EINVAL.  Synchronises the stream. */
int stq_engine_set_next(stq_engine* e, const stq_bits* next, void* hip_stream);

/* Copy the loop's state to the host and synchronise the stream (for checkpoints,
 * logging and tests; not needed to run the loop).  Any output may be NULL.
 * stored[l]: the widths the states of tensor l are held at now; next[l]: the widths the
 * next step will write (equal to stored[l] unless a decision of the default order is
 * waiting to take effect; always equal in STQ_ENGINE_ALG1_ORDER); current[l]: the
 * buffers that hold the states now; score (n doubles) and *ema: from the last decision.
 * A checkpoint is stored[], next[], the current buffers' contents, the scale arrays, the
 * parameters and *ema; stq_engine_create resumes from it, and stq_engine_set_next hands it a
 * decision that was still waiting to take effect when the checkpoint was taken (without it the
 * resumed loop keeps the stored widths until its next decision step). */
int stq_engine_read(stq_engine* e, stq_bits* stored, stq_bits* next, stq_codes* current,
                    double* score, stq_decide_state* ema, void* hip_stream);

/* Synchronise the device and free what the engine owns (not the caller's buffers). */
int stq_engine_destroy(stq_engine* e);

/* The library's own quantizer tables, for inspection (host only, no context):
 *   which 0: G[j] = fl32(2^(-j/32)), j < 511 (bits ignored)
 *   which 1: first-moment values R_b[u], u < 2^b - 1
 *   which 2: second-moment values L_b[c], c < 2^b
 *   which 3: second-moment thresholds T_b[k], k < 2^b - 1
 * Writes at most n floats to out and returns the table's length, or a negative code. */
int stq_table(int which, uint32_t bits, float* out, uint32_t n);

const char* stq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* STQ_H */
