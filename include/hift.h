/*
 * hift.h -- C ABI of the HiFT step library for AMD MI355X (gfx950).
 *
 * HiFT (hierarchical fine-tuning, arxiv 2401.15207) updates one group of layers per training
 * step: forward over the whole model, backward only from the loss down to the lowest unit of
 * the active group, weight gradients and an optimizer update for that group only, optimizer
 * state of the other groups parked in host memory (section 3, Algorithm 1).
 *
 * Conventions
 *   - Every call returns a hift_status; nothing throws across this boundary.
 *   - "device" pointers are HBM addresses of the current HIP device, "host" pointers are CPU
 *     addresses.  The library never allocates or frees device or pinned memory: the caller
 *     hands in two arenas (sizes from hift_query_bytes) and keeps them alive until
 *     hift_model_destroy.  The library owns only small host-side bookkeeping and HIP events.
 *   - Streams are hipStream_t values passed as void*; all three must have default priority.
 *   - A model is not thread-safe; calls on one model must not overlap.
 *
 * Layer units (appendix "Implementation Details", layering principle): unit 0 holds every
 * embedding table including the position table (and the embedding LayerNorm of arch 1),
 * units 1..L are the hidden layers, unit L+1 holds every head parameter including the final
 * norm.  n = L + 2.
 *
 * Canonical parameter order (fp32 values, row-major, matrices stored [out, in]); this is the
 * order of init_params_host, hift_write_params and hift_read_params:
 *   arch 0 (pre-LayerNorm decoder, learned positions, GELU, biases, causal LM loss)
 *     unit 0:   tok_emb[V,d] pos_emb[max_seq,d]
 *     unit l:   ln1_g[d] ln1_b[d] wqkv[3d,d] bqkv[3d] wo[d,d] bo[d] ln2_g[d] ln2_b[d]
 *               w1[f,d] b1[f] w2[d,f] b2[d]
 *     unit L+1: lnf_g[d] lnf_b[d] whead[V,d]
 *   arch 1 (post-LayerNorm encoder, learned positions, GELU, biases, classifier on token 0)
 *     unit 0:   tok_emb[V,d] pos_emb[max_seq,d] lne_g[d] lne_b[d]
 *     unit l:   wqkv[3d,d] bqkv[3d] wo[d,d] bo[d] ln1_g[d] ln1_b[d] w1[f,d] b1[f] w2[d,f] b2[d]
 *               ln2_g[d] ln2_b[d]
 *     unit L+1: wc[C,d] bc[C]
 *   arch 2 (RMSNorm, rotary positions on pairs (i, i+hd/2), SwiGLU, no biases, causal LM loss)
 *     unit 0:   tok_emb[V,d]
 *     unit l:   g1[d] wqkv[3d,d] wo[d,d] g2[d] wgu[2f,d] wd[d,f]
 *     unit L+1: gf[d] whead[V,d]
 *   wqkv rows are q | k | v; wgu rows are gate | up.  Heads split d into n_heads blocks of hd.
 */
#ifndef HIFT_H
#define HIFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hift_model hift_model; /* opaque, library-owned */

typedef enum {
  HIFT_OK = 0,
  HIFT_EINVAL = -1,  /* bad argument; nothing was changed */
  HIFT_ESTATE = -2,  /* call out of order (e.g. step before a schedule is set) */
  HIFT_ENOMEM = -3,  /* an arena handed in is too small */
  HIFT_EDEVICE = -4  /* a HIP call failed; hift_last_error has the HIP message */
} hift_status;

typedef enum { HIFT_BOTTOM2UP = 0, HIFT_TOP2DOWN = 1, HIFT_RANDOM = 2 } hift_strategy;
typedef enum { HIFT_ADAMW = 0, HIFT_ADAGRAD = 1, HIFT_SGD = 2, HIFT_ADAFACTOR = 3 } hift_opt_kind;
enum { HIFT_ARCH_PRELN_DECODER = 0, HIFT_ARCH_POSTLN_ENCODER = 1, HIFT_ARCH_RMS_ROPE_DECODER = 2 };
enum { HIFT_F32 = 0, HIFT_BF16 = 1 };
enum { HIFT_KIND_MATRIX = 0, HIFT_KIND_GAIN = 1, HIFT_KIND_BIAS = 2 };

typedef struct {
  int32_t arch;          /* HIFT_ARCH_* */
  int32_t n_layers;      /* L hidden layers */
  int32_t d_model;       /* d; multiple of n_heads; d / n_heads even */
  int32_t n_heads;
  int32_t d_ffn;         /* f */
  int32_t vocab;         /* V */
  int32_t max_seq;       /* rows of the position table (arch 0, 1); upper bound of seq for arch 2 */
  int32_t n_classes;     /* C (arch 1 only) */
  float norm_eps;
  float rope_base;       /* arch 2 */
  int32_t dtype;         /* HIFT_F32: all arithmetic and storage fp32.
                            HIFT_BF16: bf16 weights/activations with fp32 accumulation and fp32
                            master weights (appendix "Mixing Precision", adapted mixed precision) */
  int32_t state_on_host; /* 1: optimizer state of inactive groups lives in the pinned arena and is
                            moved per step (Algorithm 1 steps i and k); 0: all state stays in HBM */
  int32_t master_on_host; /* 1 (bf16 mode with state_on_host only): the fp32 master weights of inactive
                            groups live in the pinned arena too and travel with the state, so that HBM
                            holds the bf16 model plus one group's fp32 master (appendix "Mixing
                            Precision", the adapted mixed precision); results are identical.  0: the
                            master stays in HBM */
  int32_t no_packed_copies; /* 1: do not keep the second and third bf16 copy of the large matrices (in
                            MFMA fragment order, for the fast contraction kernel); the contractions
                            then read the row-major copy.  Saves 4 bytes per parameter, costs speed */
  int32_t tie_embeddings; /* 1 (arch 0 and 2): the output matrix is the token table (GPT-2, OPT of section
                            "Experiments"): there is no whead tensor, the shared matrix belongs to unit 0,
                            unit L+1 keeps the final norm alone, and the table's gradient is the sum over
                            its two uses */
  int32_t lora_rank;      /* > 0: low-rank adapters of this rank on the query and value projections of every hidden
                            layer (the LoRA baseline that section "Wallclock Time Efficiency" sets beside HiFT):
                            W + (lora_alpha / lora_rank) B A.  Such a model is trained with hift_lora_step only.
                            A multiple of 8 in bf16 mode */
  float lora_alpha;
  int32_t unfused;        /* 0: every fusion the shapes allow.  HIFT_UNFUSED_* bits keep the separate kernels instead
                            (same results within rounding; for comparison and for tests of the separate kernels) */
} hift_config;
/* hift_config.unfused.  EPILOGUES: rotary embedding, gated activation / GELU and their backward run as kernels of
 * their own after the contraction instead of in its epilogue.  ATTENTION: scores, softmax and the product with v
 * as separate contractions and a softmax kernel instead of the fused attention kernels.  NORM: RMS normalisation
 * as a kernel of its own instead of folded into the contraction that consumes it.  HIFT_UNSHARED_LAST_ROUND: the
 * tiles of a contraction's last, partial round are not shared between workgroups. */
enum { HIFT_UNFUSED_EPILOGUES = 1, HIFT_UNFUSED_ATTENTION = 2, HIFT_UNFUSED_NORM = 4, HIFT_UNSHARED_LAST_ROUND = 8 };

typedef struct {
  int32_t kind;        /* hift_opt_kind */
  double lr;           /* hyper-parameters are doubles so that 1 - beta and the bias corrections */
  double beta1, beta2; /* are formed from the caller's values before rounding to fp32 (AdamW) */
  double eps;          /* AdamW (1e-8 usual) and AdaGrad (1e-10 usual) */
  double weight_decay; /* applied to tensors with two or more dimensions only; AdamW: decoupled,
                          AdaGrad / SGD: added to the gradient */
  double momentum;     /* SGD; 0 = plain SGD, which keeps no state and moves no bytes */
} hift_opt;
/* HIFT_ADAFACTOR (section "Memory Efficiency Analysis" lists it among the optimizers): Shazeer and Stern
 * 2018, Algorithm 4 without momentum, with the caller's lr as the step size (no relative step, no
 * parameter scaling); epsilon_1 = 1e-30, clipping threshold 1, beta2_t = 1 - t^-0.8 with t the group's own
 * update count; matrices keep one statistic per row and per column, vectors one per element; uses lr and
 * weight_decay only.  The statistics of all groups stay in HBM (rows + cols floats per matrix), so nothing
 * moves between host and device. */

typedef struct {
  const int32_t* tokens; /* device, [batch, seq], each in [0, vocab) */
  const int32_t* labels; /* device; arch 0/2: [batch, seq], target of each position or -1 for none
                            (a causal LM batch has labels[b,s] = tokens[b,s+1] and -1 at the end);
                            arch 1: [batch], class of each sequence */
  int32_t batch, seq;
} hift_batch;

typedef struct {
  char name[32];
  int32_t unit;    /* layer unit that owns the tensor */
  int32_t kind;    /* HIFT_KIND_* ; weight decay applies to HIFT_KIND_MATRIX only */
  int64_t offset;  /* first element in the canonical flat order */
  int64_t rows, cols; /* cols = 1 for vectors */
} hift_tensor_info;

/* Section 3 "Notation": k = n/m if m divides n, otherwise floor(n/m)+1.  Pure host integer
 * helpers, usable without a GPU. */
hift_status hift_group_count(int32_t n_units, int32_t m, int32_t* k_out);
/* Visiting order of k groups (section 3.1 and Algorithm 1 initialisation).  Group ids are
 * positions in model order (group 0 holds the embeddings); the strategy only fixes the order.
 * random: Fisher-Yates from the top index down with SplitMix64 draws from `seed`, fixed for the
 * whole run.  order_out: host, k entries. */
hift_status hift_group_order(int32_t k, hift_strategy s, uint64_t seed, int32_t* order_out);

/* Parameter layout of a configuration.  hift_tensor_count gives the number of tensors and the
 * total number of parameters; hift_tensor_at fills the description of tensor `index`. */
hift_status hift_tensor_count(const hift_config* cfg, int32_t* n_tensors, int64_t* n_params);
hift_status hift_tensor_at(const hift_config* cfg, int32_t index, hift_tensor_info* out);

/* Sizes of the two arenas a model of this shape needs for batches of at most max_batch
 * sequences of at most max_seq tokens, grouped m units per group (the gradient buffer and the
 * three state slots are sized for the largest group). */
hift_status hift_query_bytes(const hift_config* cfg, const hift_opt* opt, int32_t m,
                             int32_t max_batch, int32_t max_seq,
                             size_t* device_bytes, size_t* pinned_host_bytes);

/* Where the memory goes (appendix "Memory Analysis" and the tables of appendix "Mixing Precision":
 * #Para, #Gra, #Sta, #PGS, residual states, total).  All figures in bytes.  Host-only arithmetic,
 * usable without a GPU.
 *   device_*: this library's device arena by purpose.  master = fp32 weights resident in HBM (all of
 *   them, or three group-sized slots when master_on_host); forward = the bf16 model; packed = the
 *   fragment-order copies; grad = one fp32 buffer for the largest group; state = optimizer state in HBM
 *   (three group-sized slots, or all of it); activations = everything the forward keeps for the
 *   backward; workspace = backward temporaries, tables, reduction scratch.
 *   para/gra/sta/pgs/residual/total: the same bytes in the paper's columns (para = master + forward +
 *   packed, residual = activations + workspace).
 *   zeta_*: the closed forms for fp32 AdamW: zeta1 = 4 bytes x parameters, zeta_fpft = 4 zeta1,
 *   zeta_hift = (k+3)/k zeta1 (average over equal groups), zeta_hift_peak = zeta1 + 12 bytes x
 *   parameters of the largest group; peak_trainable = parameters of the largest group. */
typedef struct {
  uint64_t device_master, device_forward, device_packed, device_grad, device_state, device_activations,
      device_workspace, device_total, pinned_total;
  uint64_t para, gra, sta, pgs, residual, total;
  uint64_t n_params, peak_trainable;
  int32_t k, reserved;
  double zeta1, zeta_fpft, zeta_hift, zeta_hift_peak;
} hift_memory;
hift_status hift_memory_report(const hift_config* cfg, const hift_opt* opt, int32_t m, int32_t max_batch,
                               int32_t max_seq, hift_memory* out);

/* Build a model inside the caller's arenas (Algorithm 1 "Require": model M, optimizer P).
 *   init_params_host  host, fp32, canonical order, n_params values; copied.  May be NULL: all
 *                     parameters start at zero and the caller fills them with hift_write_params.
 *   device_arena      device, 256-byte aligned, device_bytes long
 *   pinned_arena      host, page-locked, pinned_bytes long, zero-filled by the library
 *                     (may be NULL when pinned_host_bytes is 0)
 *   streams           compute, host-to-device, device-to-host
 * Optimizer state starts at zero.  Errors: HIFT_EINVAL (bad shape), HIFT_ENOMEM, HIFT_EDEVICE. */
hift_status hift_model_create(const hift_config* cfg, const hift_opt* opt, int32_t m,
                              int32_t max_batch, int32_t max_seq, const float* init_params_host,
                              void* device_arena, size_t device_bytes, void* pinned_arena,
                              size_t pinned_bytes, void* compute_stream, void* h2d_stream,
                              void* d2h_stream, hift_model** out);
/* The same with the pinned arena handed in as n_chunks separately allocated page-locked blocks (a host may
 * refuse one block of 50 or 100 GB and still grant it in pieces; the 13B-shaped model with AdamW parks 104 GB
 * of state: Algorithm 1 steps i and k).  pinned_chunks / pinned_chunk_bytes: host arrays of n_chunks pointers
 * and sizes; every chunk 16-byte aligned and a multiple of 16 bytes long; the sizes must add up to at least
 * pinned_host_bytes of hift_query_bytes; chunks beyond that are not touched.  The library treats the chunks as
 * one range in the order given and splits a transfer where a chunk ends.  Results are identical. */
hift_status hift_model_create_chunked(const hift_config* cfg, const hift_opt* opt, int32_t m,
                                      int32_t max_batch, int32_t max_seq, const float* init_params_host,
                                      void* device_arena, size_t device_bytes, void* const* pinned_chunks,
                                      const size_t* pinned_chunk_bytes, int32_t n_chunks, void* compute_stream,
                                      void* h2d_stream, void* d2h_stream, hift_model** out);

/* Grouping and visiting order (Algorithm 1 initialisation and steps c, d).  m may be any value
 * whose largest group fits the gradient buffer and state slots sized at creation, else
 * HIFT_ENOMEM.  Resets the step counter t to 0.  Optimizer state is kept, and with it each unit's count of
 * updates so far (the t of AdamW's bias correction: counted per unit of parameters, not per training step),
 * so a unit goes on from where it was under the new grouping.  k_out receives the number of groups. */
hift_status hift_set_group_schedule(hift_model* mdl, hift_strategy s, int32_t m, uint64_t seed,
                                    int32_t* k_out);
/* Group visited at step t (1-based): order[(t-1) mod k]. */
hift_status hift_schedule_group_at(const hift_model* mdl, int64_t t, int32_t* group_id_out);
/* Units [unit_lo, unit_hi) of a group. */
hift_status hift_group_units(const hift_model* mdl, int32_t group_id, int32_t* unit_lo,
                             int32_t* unit_hi);

/* One HiFT step (Algorithm 1 steps e to k) on one batch: forward over all units; backward from
 * the loss down to the lowest unit of group `group_id`; weight gradients of that group; its
 * optimizer state brought to HBM (prefetched during the previous step when group_id is the
 * scheduled one, fetched synchronously otherwise); optimizer update; state sent back.
 * Parameters outside the group are not written.  The work is queued on the three streams;
 * if loss_out (host) is not NULL the call waits for the compute stream and stores the mean
 * loss.  With NULL it does not wait for the step, but it may wait (when state moves and the default copy
 * engine is in use) until the host-to-device copy queued by the previous call has finished -- at most one
 * state transfer's time, normally over long before: a copy submitted while the copy engine still has a
 * backlog is run by the runtime as a full-grid kernel, which starves the step's own kernels.
 * The batch's buffers must be complete on the compute stream's timeline: the caller orders the compute
 * stream after whatever wrote them (the Python binding does this against torch's current stream).
 * Errors: HIFT_ESTATE without a schedule; HIFT_EINVAL for group_id outside [0,k), batch or seq
 * above the maxima, seq above the position table.  Token ids are not range-checked on the
 * host: an id outside [0, vocab) is clamped by the kernels. */
hift_status hift_step(hift_model* mdl, const hift_batch* batch, int32_t group_id, float* loss_out);

/* Learning rate used by following steps.  The caller applies its schedule when
 * hift_cycle_index changes (Algorithm 1: the rate moves only after all layers were updated). */
hift_status hift_set_lr(hift_model* mdl, double lr);
/* Delayed learning-rate update (section 3): the rate changes only after every group has been updated
 * once, i.e. the scheduler advances once per sweep.  Rate in force during cycle c (c = completed sweeps):
 * HIFT_LR_CONSTANT: base_lr.  HIFT_LR_LINEAR (warm-up then linear decay, the schedule of the paper's
 * hyper-parameter tables): base_lr c / warmup while c < warmup, afterwards
 * base_lr max(0, (total - c) / (total - warmup)).  hift_lr_at_cycle is a pure host helper. */
enum { HIFT_LR_CONSTANT = 0, HIFT_LR_LINEAR = 1 };
hift_status hift_lr_at_cycle(int32_t kind, double base_lr, int64_t warmup_cycles, int64_t total_cycles,
                             int64_t cycle, double* lr_out);
hift_status hift_set_lr_schedule(hift_model* mdl, int32_t kind, double base_lr, int64_t warmup_cycles,
                                 int64_t total_cycles);
/* n_steps steps of Algorithm 1, continuing from the model's step count: the i-th step of this call
 * takes batches[i mod n_batches], the group the schedule visits next, and, if a schedule was set with
 * hift_set_lr_schedule, the rate of its cycle.  batches: host array of descriptors of device buffers.
 * losses_out: host, n_steps floats, or null (then no step waits for the GPU). */
hift_status hift_train(hift_model* mdl, const hift_batch* batches, int32_t n_batches, int64_t n_steps,
                       float* losses_out);
/* Checkpoint: step count, visiting order, per-unit update counts, learning-rate schedule, fp32 master
 * weights, optimizer state of every group (wherever it lives) and Adafactor statistics, into / out of a
 * host buffer of hift_checkpoint_bytes bytes.  A run that loads a checkpoint into a model created with
 * the same configuration, optimizer kind and buffer sizes continues exactly as the saved one would have
 * (bit-identical: no kernel of the step sums in an order that depends on timing).
 * Both calls wait for the streams.  Errors: HIFT_EINVAL for a foreign, mismatching or damaged checkpoint
 * (checked completely before the model is changed: a failed load leaves it as it was), HIFT_ENOMEM for a
 * short buffer. */
hift_status hift_checkpoint_bytes(const hift_model* mdl, size_t* bytes);
hift_status hift_checkpoint_save(hift_model* mdl, void* host_buffer, size_t bytes);
hift_status hift_checkpoint_load(hift_model* mdl, const void* host_buffer, size_t bytes);
/* Steps taken since the schedule was set, and completed sweeps floor(t / k). */
hift_status hift_cycle_index(const hift_model* mdl, int64_t* steps_done, int64_t* cycles_done);

/* Low-rank adapters (hift_config.lora_rank = r > 0).  The comparison of section "Wallclock Time Efficiency": a LoRA step
 * runs the whole forward pass and the activation-gradient chain down to the first hidden layer, forms the gradients of
 * the adapters only, and updates them with AdamW (the optimizer handed to hift_model_create; no state leaves HBM: the
 * adapters are 4 r d values per layer).  Adapter parameters, canonical order, fp32: for every hidden layer
 * A_q [r, d], A_v [r, d], B_q [d, r], B_v [d, r]; hift_lora_param_count gives their number.  They start at zero.
 *   hift_lora_write / hift_lora_read: all adapters from / to host memory; which = 0 master, 1 the values the forward
 *     pass uses, 2 / 3 AdamW's first / second moment.  Both wait for the streams.
 *   hift_lora_step: one step on one batch; loss_out as for hift_step.  The base parameters are never written.
 * Errors: HIFT_ESTATE on a model without adapters (and hift_step on a model with them), HIFT_EINVAL for counts that do
 * not match. */
hift_status hift_lora_param_count(const hift_config* cfg, int64_t* n);
hift_status hift_lora_write(hift_model* mdl, const float* src_host, size_t src_count);
hift_status hift_lora_read(hift_model* mdl, int32_t which, float* dst_host, size_t dst_count);
hift_status hift_lora_step(hift_model* mdl, const hift_batch* batch, float* loss_out);

/* Copy parameters of units [unit_lo, unit_hi) to / from host memory in canonical order.
 * which = 0: fp32 master values.  which = 1 (read only): the values the forward pass uses
 * (bf16 widened to fp32 in bf16 mode).  Waits for all three streams first.
 * dst_count / src_count is the number of floats the buffer holds and must match exactly. */
hift_status hift_read_params(hift_model* mdl, int32_t unit_lo, int32_t unit_hi, int32_t which,
                             float* dst_host, size_t dst_count);
hift_status hift_write_params(hift_model* mdl, int32_t unit_lo, int32_t unit_hi,
                              const float* src_host, size_t src_count);
/* hift_write_params with the values already in device memory (src_device: device, fp32, caller-owned, complete
 * before the call): models of tens of GB are initialised without a round trip through the host. */
hift_status hift_write_params_device(hift_model* mdl, int32_t unit_lo, int32_t unit_hi,
                                     const float* src_device, size_t src_count);
/* Adafactor only: the statistics of tensor `tensor_index` (hift_tensor_at order): rows then cols floats
 * for a matrix, rows floats for a vector.  dst: host.  Waits for the streams. */
hift_status hift_read_factored_state(hift_model* mdl, int32_t tensor_index, float* dst, size_t dst_count);

/* Optimizer state of units [unit_lo, unit_hi), slot 0 (AdamW first moment / AdaGrad accumulator /
 * SGD momentum buffer) or slot 1 (AdamW second moment), wherever it currently lives. */
hift_status hift_read_state(hift_model* mdl, int32_t unit_lo, int32_t unit_hi, int32_t slot,
                            float* dst_host, size_t dst_count);

/* Bytes of optimizer state queued host-to-device and device-to-host so far (0 for plain SGD:
 * section 4.3 "Wallclock Time Efficiency", no state means no traffic). */
hift_status hift_transfer_stats(hift_model* mdl, uint64_t* h2d_bytes, uint64_t* d2h_bytes);

/* Per-step timing of the most recent hift_step, from HIP events on the compute stream:
 * whole step, and the time between the point the optimizer was ready to run and the point its
 * state had arrived (exposed copy time).  Waits for the streams. */
hift_status hift_last_step_ms(hift_model* mdl, float* step_ms, float* exposed_copy_ms);

/* How optimizer state moves between the pinned arena and HBM (Algorithm 1 steps i and k).
 * engine 0 (default): hipMemcpyAsync on the two copy streams; the library lets at most one
 * host-to-device transfer be outstanding when it submits the next, which keeps the runtime on
 * its DMA engines.  engine 1: a copy kernel with a fixed grid of `blocks` workgroups on the copy
 * streams (for comparison; kernels that touch host memory slow concurrent kernels).  Results are
 * identical.  Waits for the streams. */
hift_status hift_set_state_copy_engine(hift_model* mdl, int32_t engine, int32_t blocks);

/* Kernel-class timing for roofline reports.  While enabled, every kernel launch of hift_step is
 * bracketed by HIP events on the compute stream.  hift_profile_read sums, for one class
 * (0 linear-layer contractions, forward and dX, that run on the packed-operand kernel,
 * 1 attention contractions, 2 row-wise/elementwise kernels, 3 optimizer, 4 all other
 * linear-layer contractions: dW, small or unaligned shapes, fp32, 5 the re-packing of the updated
 * weights; one entry of class 3 or 5 covers all launches of one step), the launches since
 * hift_profile_enable, their milliseconds, and their algorithmic work (flops for classes 0, 1
 * and 4, bytes for classes 2, 3 and 5).
 * hift_profile_read_rowwise splits class 2 by kind of kernel (kind 0 .. n-1; HIFT_EINVAL beyond the last,
 * which is how a caller finds n): embedding lookup, normalisation forward, row sums of squares, rotary
 * embedding, activation forward / backward, softmax forward / backward, cross-entropy, normalisation backward
 * (dX; gain and shift), column sums, embedding gradient, first-token gather / scatter, loss bookkeeping (the two
 * one-workgroup kernels around the cross-entropy: count of targets, mean of the row losses).  name receives a static
 * string; bytes is the algorithmic traffic: every element the kernels had to read once plus every element they
 * had to write once (section "Wallclock Time Efficiency" does not cost these steps; the figure is what an
 * HBM roofline needs). */
hift_status hift_profile_enable(hift_model* mdl, int32_t on);
hift_status hift_profile_read(hift_model* mdl, int32_t category, int64_t* launches, double* total_ms,
                              double* work);
hift_status hift_profile_read_rowwise(hift_model* mdl, int32_t kind, const char** name, int64_t* launches,
                                      double* total_ms, double* bytes);

const char* hift_last_error(void); /* message of the last failing call on this thread */
void hift_model_destroy(hift_model* mdl);

/* ---- single kernels, exposed for parity tests and roofline measurement ---------------------
 * All pointers are device pointers; `stream` is a hipStream_t.  dtype is HIFT_F32 or HIFT_BF16
 * and names the element type of the activation / weight operands. */

/* C[M,N] = op(A) op(B) (+ bias[n]) (+ R[m,n]);  a_kmajor: A(m,k) at A[m*lda + k], else at
 * A[k*lda + m]; b_kmajor: B(n,k) at B[n*ldb + k], else at B[k*ldb + n].  out_f32: C is fp32
 * whatever dtype is.  bias has A's element type, R has C's type and leading dimension.  Batched over `batch` problems with element
 * strides sa, sb, sc.  HIFT_EINVAL when a leading dimension is shorter than a row of the layout named (lda < K or M, ldb < K or N,
 * ldc < N).  This is the one contraction used for every linear layer, its dX and dW
 * (Algorithm 1 steps h and the backward step). */
hift_status hift_kernel_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t out_f32,
                             int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                             const void* B, int64_t ldb, void* C, int64_t ldc, const void* bias,
                             const void* R, int32_t batch, int64_t sa, int64_t sb, int64_t sc,
                             void* stream);

/* The forward and dX contractions of large layers read the weight operand from a copy packed in
 * the register order of the matrix instruction (1 KB blocks: block (nb, kk), lane l holds
 * B[nb*32 + pi(l%32)][kk*16 + (l/32)*8 .. +7], pi = the row index with bits 2 and 3 exchanged, which
 * makes eight consecutive output columns land in one lane; rows padded to a multiple of 256).
 * hift_kernel_packed_bytes: size of that copy for a [N, K] operand, 0 if it cannot be packed
 * (needs N >= 256 and K a multiple of 32).  hift_kernel_pack_b: builds it from bf16 B given
 * k-major (B(n,k) at B[n*ldb + k], ldb >= K) or transposed (at B[k*ldb + n], ldb >= N; HIFT_EINVAL for a shorter ldb: the
 * library cannot see the size of the caller's array, so a wrong layout flag with a long enough ldb reads past it).  hift_kernel_gemm_packed:
 * C[M,N] = A . B^T (+bias)(+R) with bf16 k-major A; HIFT_EINVAL for problems the kernel does
 * not take (fewer than 200 tiles of 128x256, unaligned operands). */
hift_status hift_kernel_packed_bytes(int64_t N, int64_t K, size_t* bytes);
hift_status hift_kernel_pack_b(int32_t b_kmajor, int64_t N, int64_t K, const void* B, int64_t ldb,
                               void* Bp, void* stream);
hift_status hift_kernel_gemm_packed(int32_t out_f32, int64_t M, int64_t N, int64_t K, const void* A,
                                    int64_t lda, const void* Bp, void* C, int64_t ldc,
                                    const void* bias, const void* R, void* stream);

/* hift_kernel_gemm_packed with a work space: when the tiles of the problem leave a last round over the
 * 256 compute units in which at most half of them would have a tile, each of those tiles is shared by 2
 * to 4 workgroups that take consecutive shares of K and are summed, in a fixed order, by whichever of
 * them finishes last.  workspace: device, hift_kernel_packed_workspace_bytes() bytes, 16-byte aligned;
 * its first 1 KB must be zero before the first call and every call leaves it zero; calls that share a
 * work space must not overlap.  Same result as without it up to the order of the fp32 sums. */
hift_status hift_kernel_packed_workspace_bytes(size_t* bytes);
hift_status hift_kernel_gemm_packed_ws(int32_t out_f32, int64_t M, int64_t N, int64_t K, const void* A,
                                       int64_t lda, const void* Bp, void* C, int64_t ldc,
                                       const void* bias, const void* R, void* workspace,
                                       size_t workspace_bytes, void* stream);

/* hift_kernel_gemm_packed_ws for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the work space is an array built into the library, 32 MiB + 1 KiB
 * on every GPU the library is loaded on, held until the process ends.  Allocates nothing; the first call on a GPU
 * looks the array's address up.  Same arguments, result and errors as hift_kernel_gemm_packed_ws without the work
 * space; HIFT_EINVAL also if the problem's shared round would need more than the array holds.  Every call on a GPU
 * uses that GPU's one array (its counters are cleared by a small kernel on `stream` first): calls that overlap on
 * one GPU, on different streams or from different threads, race. */
hift_status hift_kernel_gemm_packed_static(int32_t out_f32, int64_t M, int64_t N, int64_t K, const void* A,
                                           int64_t lda, const void* Bp, void* C, int64_t ldc, const void* bias,
                                           const void* R, void* stream);

/* A linear layer of the RMSNorm / rotary / gated-FFN decoder with the elementwise step that follows it
 * done in the contraction's epilogue (forward and backward of Algorithm 1 step h; bf16).  A: device
 * [M, K] (row stride lda); W: device [N, K] bf16, contiguous; packed_scratch: device,
 * hift_kernel_packed_bytes(N, K) bytes, receives W in fragment order with its 32-row blocks arranged
 * for the epilogue.
 *   HIFT_EPILOGUE_SWIGLU: W = gate | up (N = 2 f).  C: device [M, N] or NULL, the rounded
 *     pre-activations; aux: device [M, f], receives silu(gate) * up from the rounded pre-activations.
 *   HIFT_EPILOGUE_ROPE: W = q | k | v with heads of width 128.  C: device [M, N]; columns below
 *     rot_cols are rotated pairwise (i, i + 64 inside a head) by the angle of position row % seq;
 *     cos_sin: device fp32 [>= seq, 64, 2] (cos, sin).  aux is ignored.
 *   HIFT_EPILOGUE_SWIGLU_BWD: A . W^T is the gradient of the gated activation, [M, N], and is not
 *     stored; aux: device [M, 2 N], the forward's pre-activations gate | up (read only); C: device
 *     [M, 2 N], receives d gate | d up.
 * N a multiple of 256 (of 8 for the backward epilogue); HIFT_EINVAL for problems the packed-operand
 * kernel does not take. */
enum { HIFT_EPILOGUE_SWIGLU = 1, HIFT_EPILOGUE_ROPE = 2, HIFT_EPILOGUE_SWIGLU_BWD = 3 };
hift_status hift_kernel_linear_fused(int32_t epilogue, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                     const void* W, void* packed_scratch, void* C, void* aux,
                                     const float* cos_sin, int32_t seq, int64_t rot_cols, void* stream);

/* The RMS normalisation in front of such a layer done by the layer itself (forward of Algorithm 1
 * step h; bf16): y = (x / rms(x) * gain) . W^T is computed as (1 / rms(x)) (x . (W gain)^T).
 *   hift_kernel_gemm_packed_rowsq: hift_kernel_gemm_packed with bf16 C (N a multiple of 256, R optional)
 *     that also leaves the sums of squares of the values it stored: rowsq, device fp32 [M, N / 64], one
 *     partial per row and 64-column strip.
 *   hift_kernel_row_sumsq: the same quantity for rows written by something else: x device bf16
 *     [rows, d] contiguous, d a multiple of 8; out device fp32 [rows, n]: out[r][0] = sum of squares,
 *     the other n - 1 entries of the row zero.
 *   hift_kernel_linear_norm_fused: hift_kernel_linear_fused (SWIGLU or ROPE) on rows A that are not
 *     normalised yet.  gain: device bf16 [K], multiplied into the packed copy of W (each product rounded
 *     once); rowsq: device fp32 [M, K / 64], 16-byte aligned, a row's entries add up to its sum of
 *     squares; every accumulator of row r is multiplied by 1 / sqrt(sum_r / K + norm_eps) before the
 *     epilogue proper; stats: device fp32 [M, 2] or NULL, receives (0, that factor) per row, what
 *     hift_kernel_norm_fwd leaves for the backward pass.  K a multiple of 512, at most 6144.  gain and rowsq both
 *     NULL: exactly hift_kernel_linear_fused.
 * workspace (the first and the last of the three): NULL, or a work space as hift_kernel_gemm_packed_ws
 * takes it (hift_kernel_packed_workspace_bytes() bytes, same rules), with the same effect. */
hift_status hift_kernel_gemm_packed_rowsq(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                          const void* Bp, void* C, int64_t ldc, const void* R,
                                          float* rowsq, void* workspace, void* stream);
hift_status hift_kernel_row_sumsq(int64_t rows, int32_t d, const void* x, int32_t n, float* out, void* stream);
hift_status hift_kernel_linear_norm_fused(int32_t epilogue, int64_t M, int64_t N, int64_t K, const void* A,
                                          int64_t lda, const void* W, const void* gain, void* packed_scratch,
                                          void* C, void* aux, const float* cos_sin, int32_t seq,
                                          int64_t rot_cols, const float* rowsq, float norm_eps,
                                          float* stats, void* workspace, void* stream);

/* A linear layer followed by GELU (erf form), or the dX contraction through the layer after it followed by
 * GELU's derivative, with the elementwise step in the contraction's epilogue (forward and backward of
 * Algorithm 1 step h for the feed-forward block of the GELU architectures; bf16).  A: device [M, K] (row
 * stride lda); W: device [N, K] bf16, contiguous; packed_scratch as for hift_kernel_linear_fused.
 *   backward = 0: bias device bf16 [N] or NULL; C: device [M, N] or NULL, the rounded pre-activations
 *     A . W^T + bias; aux: device [M, N], receives gelu of the rounded pre-activations.
 *   backward = 1: A . W^T is the gradient of the activation and is not stored; aux: device [M, N], the
 *     forward's pre-activations (read only); C: device [M, N], receives that gradient times gelu'(pre).
 * erf is evaluated by a formula with absolute error below 1.5e-7.  N a multiple of 8; HIFT_EINVAL for
 * problems the packed-operand kernel does not take. */
hift_status hift_kernel_linear_gelu(int32_t backward, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                    const void* W, const void* bias, void* packed_scratch, void* C, void* aux,
                                    void* stream);

/* Group-local optimizer update on `count` contiguous parameters (the update inside Algorithm 1's
 * backward step): master, grad, state1, state2 fp32; compute_copy (bf16, may be NULL) receives the
 * rounded new values.  t is the group's update number (1 on its first update). */
hift_status hift_kernel_optimizer(const hift_opt* opt, int64_t count, int32_t decay, int64_t t,
                                  float* master, const float* grad, float* state1, float* state2,
                                  void* compute_copy, void* stream);

/* Attention, fused (forward and backward of Algorithm 1 step h for one layer's attention): bf16 only,
 * head_dim 64 or 128, seq a multiple of 8, buffers 16-byte aligned, else HIFT_EINVAL.
 * qkv: device [batch*seq, 3*heads*head_dim], row = q | k | v of all heads side by side (already rotated
 * where the architecture rotates).  The scale is 1/sqrt(head_dim); causal != 0 masks keys after the query.
 * Forward: ctx: device [batch*seq, heads*head_dim].  prob: device [batch, heads, seq, seq] bf16 or NULL;
 * if given it receives the probabilities, completely (zeros where masked), and ctx is the product of
 * those rounded probabilities with v; if NULL the rows are normalised once at the end instead (one pass
 * over the keys; ctx then differs from the other case in the last bf16 digit).  lse: device fp32
 * [batch*heads*seq] or NULL; if given it receives log2 of each row's sum of exponentials of the scaled
 * scores, which is all the backward needs of the softmax.
 * Backward: ctx and lse as the forward left them; dctx: device [batch*seq, heads*head_dim], gradient of
 * ctx.  Writes all of dqkv: device [batch*seq, 3*heads*head_dim] (dq, dk, dv); the probabilities and their
 * gradient are formed again tile by tile and never stored.  dsum: device fp32 [batch*heads*seq], work space
 * (receives sum_e dctx * ctx per row).  cos_sin: device fp32 [>= seq, head_dim/2, 2] (cos, sin) or NULL;
 * if given, q and k are taken to have been rotated by the rotary embedding after their projection (pairs
 * (i, i + head_dim/2), position = row within the sequence) and dq, dk are un-rotated on the way out.
 * Buffers stay the caller's; none may overlap another. */
hift_status hift_kernel_attention_fwd(int32_t batch, int32_t heads, int32_t seq, int32_t head_dim, int32_t causal,
                                      const void* qkv, void* prob, void* ctx, float* lse, void* stream);
hift_status hift_kernel_attention_bwd(int32_t batch, int32_t heads, int32_t seq, int32_t head_dim, int32_t causal,
                                      const void* qkv, const void* ctx, const float* lse, const void* dctx,
                                      float* dsum, void* dqkv, const float* cos_sin, void* stream);
/* y = norm(x) * g (+ b) over rows of width d; rms = 1: RMSNorm (b ignored).  stats: fp32 [rows,2]
 * receives mean (0 for RMSNorm) and reciprocal standard deviation. */
hift_status hift_kernel_norm_fwd(int32_t dtype, int32_t rms, int64_t rows, int32_t d, float eps,
                                 const void* x, const void* g, const void* b, void* y,
                                 float* stats, void* stream);

/* Mean cross-entropy over rows with label >= 0 and its gradient: logits [rows, V] are replaced
 * by d loss / d logits; loss_out is one device float. */
hift_status hift_kernel_cross_entropy(int32_t dtype, int64_t rows, int32_t V, void* logits,
                                      const int32_t* labels, float* row_loss_scratch,
                                      float* loss_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HIFT_H */
