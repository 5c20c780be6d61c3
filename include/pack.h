/*
 * pack.h - C ABI of the packed-training library for AMD MI355X (gfx950).
 *
 * The library implements the `pack` primitive of "Understanding and Optimizing Packed Neural
 * Network Training for Hyper-Parameter Tuning" (Liu, Krishnan, Elmore, Franklin): K independent
 * networks are joined into one network by concatenating their outputs (Section 2.2, Section 3.1);
 * when they train on the same data the K inputs are rewritten to ONE shared input (Section 3.4);
 * members with a smaller batch size train on a slice of the shared batch (Section 3.2); every
 * member keeps its own hyper-parameters (Section 2.2, task trait (a)); and all members are
 * differentiated and updated in one synchronised step (Section 2.2).  The guarantee the paper
 * states in Section 2.2 is the contract of this ABI: every member's input, output and
 * back-propagation are exactly those of the member trained alone on a dedicated device.
 *
 * One `pack_t` is one packed model resident on one GPU: the paper's `pack` + `load`.
 * `pack_read_weights` (+ `pack_read_opt_state`) followed by `pack_free` or `pack_destroy` is the
 * paper's `free` (retrieve the checkpoint, release the memory).  Members can leave and join a live
 * pack (`pack_free`, `pack_load`; Section 3.3), and an epoch over members with different batch
 * sizes is driven by `pack_schedule_*`, `pack_gather_batch` and `pack_set_batch` (Section 3.2).
 * A pack has K slots; a slot holds a member or is vacant.  Calls that name a vacant slot fail with
 * PACK_EINVAL; arrays indexed by member (lr, loss, batch) have one entry per slot and the entries
 * of vacant slots are ignored (read as 0).
 *
 * Conventions
 *   - All functions return a pack_status; nothing is thrown across the ABI.  A failing call
 *     leaves the pack unchanged.  pack_last_error() returns a thread-local description.
 *   - "dev" pointers are device memory of the GPU that was current at pack_create; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes in.  The library
 *     owns weights (fp32 master, bf16 operand copy), activations, gradients, loss/prediction
 *     buffers and the launch plan, and releases them in pack_destroy.
 *   - pack_step only enqueues work on the stream given at pack_create and does not wait for it.
 *     pack_read_* and pack_write_weights wait for that stream.
 *   - Shared batch x: row-major [B, D] for flat inputs, NHWC [B, H, W, C] for images; element type
 *     float for PACK_F32 packs, bfloat16 (upper 16 bits of a float) for PACK_BF16 packs.
 *   - labels: int32 [B], one vector shared by all members (one dataset, Section 3.4), values in
 *     [0, C_k) for every member k.
 *   - Per-member flat weight blob (always float): layers in order; PACK_LINEAR stores
 *     W[out][in] then b[out]; PACK_CONV3X3 stores W[Cout][Cin][3][3] then b[Cout].  A linear
 *     layer applied to an image sees it flattened in NHWC order.
 *   - PACK_BF16: matrix operands (x, activations, stored gradients, a per-step bf16 copy of the
 *     weights) are bfloat16; products accumulate in fp32; bias add, ReLU, softmax
 *     cross-entropy, weight gradients and the update are fp32; the master weights stay fp32.
 */
#ifndef PACK_H
#define PACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pack_ctx pack_t;

typedef enum {
    PACK_OK = 0,
    PACK_EINVAL = 1,   /* null pointer, K < 1 or > PACK_MAX_MODELS, unknown op, bad stride, batch outside [1, B] */
    PACK_ENOMEM = 2,   /* device or host allocation failed (the out-of-memory case of Section 4.2) */
    PACK_EDEVICE = 3,  /* a HIP runtime call failed */
    PACK_ESHAPE = 4,   /* layer list is not a classifier this library can run (see pack_create) */
    PACK_ELABEL = 5,   /* a label outside [0, C_k) was seen since the last pack_read_loss */
    PACK_EINDEX = 6    /* pack_gather_batch met a sample index outside the dataset since the last pack_read_loss */
} pack_status;

typedef enum {
    PACK_LINEAR = 0,    /* fully connected, with bias; `out` = output features */
    PACK_CONV3X3 = 1,   /* 3x3 convolution, zero padding 1, with bias; `out` = channels, `stride` 1 or 2 */
    PACK_RELU = 2,      /* max(z, 0); must directly follow PACK_LINEAR or PACK_CONV3X3 */
    PACK_GAP = 3,       /* global average pool over H x W */
    PACK_RES_BEGIN = 4, /* the current tensor becomes the shortcut source of a residual block */
    PACK_RES_END = 5,   /* y = relu(current + shortcut(source)); must directly follow PACK_CONV3X3.
                           shortcut = identity when shapes agree; otherwise source[b,2i,2j,c] for
                           c < Cin and 0 for the remaining channels (parameter-free) */
    /* the other activations of the paper's search space (Section 5.3, Table 3); like PACK_RELU each
       must directly follow PACK_LINEAR or PACK_CONV3X3 */
    PACK_SIGMOID = 6,   /* 1 / (1 + exp(-z)) */
    PACK_TANH = 7,      /* tanh(z) */
    PACK_LEAKY_RELU = 8 /* z > 0 ? z : 0.2 z (the paper names no slope; 0.2 is the default of the
                           framework it ran on) */
} pack_op;

typedef enum { PACK_F32 = 0, PACK_BF16 = 1 } pack_dtype;

/* Optimisers of the paper's search space (Section 5.3, Table 3).  A member's optimiser is one of its
 * hyper-parameters (Section 2.2, task trait (a)); members of one pack may differ (Table 2,
 * "Optimizer: Different").  The paper prints no update formula; the library follows the published
 * definitions of the methods it names, always with gradients taken at the pre-update weights:
 *   PACK_OPT_SGD       W <- W - lr*g
 *   PACK_OPT_MOMENTUM  acc <- mu*acc + g;  W <- W - lr*acc                    (acc starts at 0)
 *   PACK_OPT_ADAGRAD   acc <- acc + g*g;   W <- W - lr*g/sqrt(acc)            (acc starts at acc0)
 *   PACK_OPT_ADAM      m <- beta1*m + (1-beta1)*g;  v <- beta2*v + (1-beta2)*g*g;  t <- t+1;
 *                      W <- W - lr * (m/(1-beta1^t)) / (sqrt(v/(1-beta2^t)) + eps)   (m, v, t start at 0) */
typedef enum { PACK_OPT_SGD = 0, PACK_OPT_MOMENTUM = 1, PACK_OPT_ADAGRAD = 2, PACK_OPT_ADAM = 3 } pack_opt_kind;

typedef struct {
    int32_t kind;        /* pack_opt_kind */
    float mu;            /* PACK_OPT_MOMENTUM: in [0, 1) */
    float acc0;          /* PACK_OPT_ADAGRAD: initial accumulator, > 0 */
    float beta1, beta2;  /* PACK_OPT_ADAM: in [0, 1) */
    float eps;           /* PACK_OPT_ADAM: > 0 */
} pack_opt_spec;

#define PACK_MAX_MODELS 256

typedef struct {
    int32_t op;      /* pack_op */
    int32_t out;     /* output features / channels (PACK_LINEAR, PACK_CONV3X3), else ignored */
    int32_t stride;  /* PACK_CONV3X3 only: 1 or 2 */
} pack_layer;

/* One member = the paper's "training task" (Section 2.2) minus device and step count. */
typedef struct {
    const pack_layer* layers;  /* host */
    int32_t n_layers;
    int32_t batch;             /* b_k in [1, B]: the member trains on rows [0, b_k) of the shared batch */
} pack_model_spec;

typedef struct {
    int32_t B;                 /* rows of the shared batch */
    int32_t in_h, in_w, in_c;  /* flat input of D features: in_h = in_w = 1, in_c = D */
    int32_t dtype;             /* pack_dtype */
} pack_input_spec;

/* pack + load (Section 2.2): build the packed model for K members on the current device.
 * `models` and the layer arrays are host memory and are copied.  Weights are initialised from
 * `seed` (uniform in +-sqrt(6/fan_in), biases in +-1/sqrt(fan_in)); callers that need specific
 * weights use pack_write_weights.  `hip_stream` is a hipStream_t (0 = the null stream) on
 * which every later call enqueues its work.
 * The layer list must end in a PACK_LINEAR (without ReLU): its output [b_k, C_k] is the logits.
 * Errors: PACK_EINVAL, PACK_ESHAPE (unsupported op order, RES_BEGIN/RES_END mismatch, shortcut
 * shapes that neither agree nor halve, last layer not linear), PACK_ENOMEM, PACK_EDEVICE. */
pack_status pack_create(const pack_input_spec* input, const pack_model_spec* models, int32_t K,
                        uint64_t seed, void* hip_stream, pack_t** out);

/* Plan verification on the host; no GPU is involved and none is needed.  Plans the pack exactly as
 * pack_create would (same planner, made-up device addresses) and walks every matrix-product launch of the
 * plan: for the staged-tile kernels the kernels' own fetchers are run on the CPU, thread by thread and chunk
 * by chunk (prefetches beyond the reduction included), and every load is held against the definition of the
 * operands of the product the launch computes (the forward and backward passes of the members' layers,
 * Section 2.2: "as if trained alone"); for the halo kernels of the 3x3 convolutions the walk also follows
 * what is stored to LDS and read back as matrix-instruction operands.  A load of existing elements outside
 * its descriptor's window or its allocation, a load of missing elements that is not cut off by construction,
 * an operand slot holding the wrong element, a tile dealt twice or not at all is an error.
 * input_mode: pack_input_mode.  Outputs (host, may be null): launches walked, matrix-product launches on the
 * element-by-element kernels for unaligned shapes (skipped: they load by the definition itself), loads and
 * operand reads checked.
 * Errors: PACK_EINVAL (bad arguments, or a violation: pack_last_error names launch and tile), PACK_ESHAPE, PACK_ENOMEM. */
pack_status pack_plan_check(const pack_input_spec* input, const pack_model_spec* models, int32_t K, int32_t input_mode,
                            int64_t* launches_walked, int64_t* launches_skipped, int64_t* loads_checked);

/* free of ONE member of a live pack (Section 2.2 `free`; Section 3.3, Figure 3: the member that has
 * taken all its steps is freed while the others keep training).  The caller retrieves the
 * checkpoint first (pack_read_weights, pack_read_opt_state).  Slot k becomes vacant and the member's
 * device memory is released.  Weights, optimiser state and step counters of every other member are
 * carried over on the device bit for bit, so their training continues exactly as if nothing had
 * happened.  Waits for the stream.  While the call runs the pack holds its old and new buffers at
 * once.  Per-launch timing is switched off and launch indices change.
 * Errors: PACK_EINVAL (k out of range or vacant), PACK_ENOMEM, PACK_EDEVICE; the pack is unchanged then. */
pack_status pack_free(pack_t* p, int32_t k);

/* load of one more member into a live pack (Section 2.2 `load`; Section 3.3: a fresh model may join
 * the members that have not finished yet).  The member takes the lowest vacant slot, or a new
 * slot at the end (the number of slots grows by one); *k_out receives the slot.  Its weights are
 * seeded as in pack_create from (seed, slot) (use pack_write_weights / pack_write_opt_state to load a
 * checkpoint), its optimiser is PACK_OPT_SGD.  Other members as in pack_free.
 * Errors: PACK_EINVAL (null, batch outside [1, B], PACK_MAX_MODELS slots in use), PACK_ESHAPE,
 * PACK_ENOMEM, PACK_EDEVICE; the pack is unchanged then. */
pack_status pack_load(pack_t* p, const pack_model_spec* model, uint64_t seed, int32_t* k_out);

/* Re-slice the shared batch (Section 3.2): from now on the shared batch has B rows and member k
 * trains on rows [0, batch[k]).  batch: host int32 [pack_num_slots(p)].  Used when the member with
 * the largest batch has left (the next largest batch becomes the shared batch) and for the short
 * last batch of a phase.  Member state is carried over as in pack_free; a call that changes nothing
 * returns at once.  Errors: PACK_EINVAL (null, B < 1, batch[k] outside [1, B]), PACK_ENOMEM, PACK_EDEVICE. */
pack_status pack_set_batch(pack_t* p, int32_t B, const int32_t* batch);

/* Which data the members train on.  PACK_INPUT_SHARED (the default; Section 3.4): one batch and one
 * label vector for all members.  PACK_INPUT_PER_MEMBER (the "Training Data: Different" rows of the
 * paper's ablation, Section 4.7 / Table 2): every slot has its own batch; pack_step then takes x_dev as
 * [pack_num_slots][B, H, W, C] and labels_dev as [pack_num_slots][B], and member k trains on rows
 * [0, b_k) of block k.  Nothing is shared between members any more: each first layer (and, for
 * convolutions over few channels, each im2col copy) reads its own block.  Changing the mode plans the
 * pack again; member state is carried over as in pack_free.
 * Errors: PACK_EINVAL (null, unknown mode), PACK_ENOMEM, PACK_EDEVICE. */
typedef enum { PACK_INPUT_SHARED = 0, PACK_INPUT_PER_MEMBER = 1 } pack_input_mode;
pack_status pack_set_input_mode(pack_t* p, int32_t mode);

/* Number of slots K (members + vacant slots); 0 if p is null. */
int32_t pack_num_slots(const pack_t* p);

/* b_k of member k; 0 if the slot is vacant or out of range. */
int32_t pack_member_batch(const pack_t* p, int32_t k);

/* Epoch schedule for members with different batch sizes (Section 3.2: every member's progress
 * through the dataset is followed separately; step counts as in Section 3.3).  Host logic, no GPU involved.  The shared
 * batch of a step has the size of the largest batch among the members that have not yet used the
 * whole dataset and is cut, in dataset order, from the samples THAT member has not used; every other
 * unfinished member trains on the leading rows.  When the member with the largest batch has used
 * everything it leaves and the next largest batch leads.  Every member sees every sample exactly
 * once.  A phase whose samples do not divide by the batch size ends with one short shared batch.
 * pack_schedule_create: n_samples >= 1; batch: host int32 [K], each >= 1.
 * pack_schedule_next: writes the sample indices of the next shared batch into idx_host (host int64,
 *   room for max(batch) entries), their number into *rows, the number of leading rows each member
 *   trains on into rows_k (host int32 [K]; 0 = the member has finished) and, if lead is not null, the
 *   member whose batch size rules the phase.  After the last step of the epoch it returns PACK_OK
 *   with *rows = 0.
 * pack_schedule_used: samples each member has trained on so far (host int64 [K]).
 * Errors: PACK_EINVAL, PACK_ENOMEM. */
typedef struct pack_schedule pack_schedule_t;
pack_status pack_schedule_create(int64_t n_samples, const int32_t* batch, int32_t K, pack_schedule_t** out);
pack_status pack_schedule_next(pack_schedule_t* s, int64_t* idx_host, int32_t* rows, int32_t* rows_k, int32_t* lead);
pack_status pack_schedule_used(const pack_schedule_t* s, int64_t* used_host);
void pack_schedule_destroy(pack_schedule_t* s);

/* Assemble a shared batch from a dataset resident on the device (Section 3.2: the shared batches of
 * later phases are cut from the samples not yet used, which are not contiguous):
 * x_out[r] = data[idx[r]] and labels_out[r] = labels_all[idx[r]] for r < rows.  All pointers are
 * device memory; data: [n_samples, H, W, C] of the pack's dtype; labels_all: int32 [n_samples];
 * idx: int64 [rows]; x_out: room for B rows (16-byte aligned, as pack_step requires); labels_out:
 * int32 [B].  rows in [0, B]; rows beyond `rows` are left as they are.  Enqueues one kernel on the
 * pack's stream.  An index outside [0, n_samples) gives a row of zeros with label -1 (ignored by the
 * loss) and makes the next pack_read_loss return PACK_EINDEX.
 * Errors: PACK_EINVAL (null, rows outside [0, B], misaligned pointer), PACK_EDEVICE. */
pack_status pack_gather_batch(pack_t* p, const void* data_dev, const int32_t* labels_all_dev, int64_t n_samples,
                              const int64_t* idx_dev, int32_t rows, void* x_out_dev, int32_t* labels_out_dev);

/* ---- pack-aware hyper-parameter search (Section 5): host logic, no GPU involved -------------------
 * A configuration is a row of D table indices (for the paper's Table 3: batch size, optimiser, learning
 * rate, activation); categorical[j] != 0 marks a dimension without an order.  Every random choice is an
 * argument, so a search can be replayed.  Groups are returned as one group number per configuration,
 * numbered in the order the groups were formed.
 *
 * pack_config_distance: Section 5.2: numeric dimensions contribute |index difference|, categorical ones
 *   0 if equal else 1; the contributions are added (the text's worked example: batch size 20 -> 40 is
 *   four index steps, plus a different optimiser: 5).  Returns -1 on a null argument.
 * pack_opt_knn: Section 5.2, the nearest-neighbour heuristic.  feats: host int32 [T][D]; need: host
 *   uint64 [T], the device memory each configuration takes as a member (pack_estimate_bytes);
 *   capacity: the memory available; threshold: the similarity threshold (largest distance to the
 *   centroid at which a configuration may still join); draws: host double [T] in [0, 1), draw j picks
 *   the centroid of group j as element floor(u * remaining) of the configurations not yet grouped, in
 *   list order.  Candidates join nearest first (list order on ties) while they fit; one that does not
 *   fit is passed over.  A configuration larger than the capacity forms a group of its own.
 * pack_opt_random: Section 5.3 "Random Pack": the configurations in the order of perm (host int32 [T],
 *   a permutation), m per group.
 * pack_opt_batchsize: Section 5.3 "Batch-size Pack": batch: host int32 [T]; only equal values share a
 *   group; groups are filled in list order until the next configuration does not fit.
 * pack_hyperband_plan: the brackets of Hyperband (Section 5.1, Algorithm 1, with the bracket sizes of the
 *   Hyperband paper it cites): bracket j has rungs_out[j] rungs; the rungs of all brackets follow each
 *   other in n_out / r_out (configurations alive in the rung, resource units each has been trained for
 *   when the rung ends).  capacity: entries available in n_out and r_out.
 * pack_halving_keep: the `keep` smallest of n losses, the earlier on ties, as increasing indices.  A NaN loss
 *   (a diverged configuration) ranks after every number, +inf included, so it never displaces a finite one.
 * Errors: PACK_EINVAL. */
int32_t pack_config_distance(const int32_t* a, const int32_t* b, const uint8_t* categorical, int32_t n_dims);
pack_status pack_opt_knn(const int32_t* feats, const uint8_t* categorical, int32_t T, int32_t D, const uint64_t* need,
                         uint64_t capacity, int32_t threshold, const double* draws, int32_t* group_out, int32_t* n_groups);
pack_status pack_opt_random(int32_t T, int32_t m, const int32_t* perm, int32_t* group_out, int32_t* n_groups);
pack_status pack_opt_batchsize(const int32_t* batch, int32_t T, const uint64_t* need, uint64_t capacity,
                               int32_t* group_out, int32_t* n_groups);
pack_status pack_hyperband_plan(int32_t R, int32_t eta, int32_t* n_out, int32_t* r_out, int32_t* rungs_out,
                                int32_t capacity, int32_t* n_brackets);
pack_status pack_halving_keep(const float* loss, int32_t n, int32_t keep, int32_t* idx_out);

/* The memory model of pack_opt (the paper finds the limit by running out of memory, Section 5.2; here
 * it is computed): bytes of device memory a member with this layer list, batch size and optimiser adds
 * to a pack - parameters (master, gradient, operand copy, optimiser state), activations and their
 * gradients - not counting what members share (im2col copy of the input, workspace of split
 * reductions, problem tables).  0 if the specification is invalid. */
size_t pack_estimate_bytes(const pack_input_spec* input, const pack_model_spec* model, int32_t opt_kind);

/* Measuring aid (Section 4.1 reports every figure on one named device; a rate is only meaningful
 * beside what that device delivers): what this GPU sustains on the simplest code of each kind, timed
 * with events on `stream` (host handle of a HIP stream, or null for the default stream).
 *   PACK_CEILING_HBM_COPY: a streaming copy of 1 GiB, bytes read + bytes written, in GB/s;
 *   PACK_CEILING_MFMA_BF16 / _FP32: a loop of 32x32 matrix instructions on register operands, the shape
 *     the GEMM kernels use, fp32 accumulation, in TFLOP/s.
 * Allocates its own buffers (2 GiB for the copy) and frees them before it returns; takes a few
 * milliseconds.  value_out: host double.  PACK_EINVAL on an unknown `what` or a null pointer,
 * PACK_EDEVICE if a HIP call fails (out of memory included). */
enum { PACK_CEILING_HBM_COPY = 0, PACK_CEILING_MFMA_BF16 = 1, PACK_CEILING_MFMA_FP32 = 2 };
pack_status pack_measure_ceiling(int32_t what, void* stream, double* value_out);

/* load a member's weights (Section 2.2 `load`): host_src holds pack_num_params(p, k) floats in
 * the blob layout above.  For PACK_BF16 the bf16 operand copy is refreshed too.
 * Errors: PACK_EINVAL (k out of range, n_floats mismatch), PACK_EDEVICE. */
pack_status pack_write_weights(pack_t* p, int32_t k, const float* host_src, size_t n_floats);

/* One synchronised training step of all K members (Section 2.2; shared input Section 3.4; batch
 * slices Section 3.2): forward, mean softmax cross-entropy over each member's own rows, backward,
 * and W <- W - lr[k] * dW for every parameter of member k, with gradients taken at the
 * pre-update weights.  x_dev: device, 16-byte aligned, [B, H, W, C] of the pack's dtype; labels_dev: device int32
 * [B] (K blocks of that shape each after pack_set_input_mode(PACK_INPUT_PER_MEMBER)); lr_host: host
 * float [K], copied during the call.  Enqueues only.
 * Errors: PACK_EINVAL (null argument), PACK_EDEVICE (launch failure). */
pack_status pack_step(pack_t* p, const void* x_dev, const int32_t* labels_dev, const float* lr_host);

/* pack_step for callers that may not allocate device memory while they run: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The same step with the same kernels and the same
 * bits as pack_step; the only difference is where the partial sums of split weight gradients go: not into
 * the workspace the pack allocated at creation but into a scratch array that is part of the library's code
 * object (file-scope device memory, pack_static_scratch_bytes() = 128 MiB, 0.04 % of the card; every GPU
 * the library runs on holds its own copy until the process ends).  The call allocates and frees nothing,
 * on the device or through any library; the first call on a device looks the array's address up.
 * A pack whose split weight gradients need more than the array holds (pack_workspace_bytes(p)) is rejected
 * with PACK_ENOMEM and nothing is launched; the five reference configurations need at most 113 MB.  Launch
 * timing must be off (PACK_EINVAL otherwise: events are allocations).  All packs of a process share the
 * array of their GPU: a step overwrites what the previous one left there and needs nothing cleared, but
 * two steps that overlap in time on one GPU (different streams or threads) race on it; keep such steps on
 * one stream, or use pack_step.
 * Errors: PACK_EINVAL, PACK_ENOMEM, PACK_EDEVICE. */
pack_status pack_step_static(pack_t* p, const void* x_dev, const int32_t* labels_dev, const float* lr_host);
size_t pack_static_scratch_bytes(void);
/* Bytes of scratch one step of this pack needs for the partial sums of split weight gradients. */
size_t pack_workspace_bytes(const pack_t* p);

/* Choose member k's optimiser (default: PACK_OPT_SGD).  Resets the member's optimiser state to its
 * starting values and its step counter to 0; the weights are untouched.  Fields that the chosen
 * kind does not use are ignored.  Waits for the stream.  The learning rate stays the per-step
 * argument of pack_step.
 * Errors: PACK_EINVAL (null, k out of range, unknown kind, parameter outside its range), PACK_ENOMEM. */
pack_status pack_set_optimizer(pack_t* p, int32_t k, const pack_opt_spec* spec);

/* The optimiser part of free's checkpoint (Section 2.2 keeps an optimiser's state with its model): state
 * array `slot` of member k in the blob layout of the weights (slot 0: momentum / Adagrad accumulator
 * or Adam's first moment; slot 1: Adam's second moment) and, if `steps` is not null, the number of
 * steps the optimiser has taken.  pack_write_opt_state restores both (the load of a checkpoint).
 * Errors: PACK_EINVAL (null, k out of range, n_floats mismatch, slot the member's optimiser does not have). */
pack_status pack_read_opt_state(pack_t* p, int32_t k, int32_t slot, float* host_dst, size_t n_floats, int64_t* steps);
pack_status pack_write_opt_state(pack_t* p, int32_t k, int32_t slot, const float* host_src, size_t n_floats, int64_t steps);

/* Loss of each member at the last step, evaluated at that step's pre-update weights.
 * host_dst: float [K].  Waits for the stream.  Returns PACK_ELABEL (and still fills host_dst)
 * if any step since the previous pack_read_loss met a label outside [0, C_k); such rows
 * contribute nothing to loss or gradients and index no memory.  Returns PACK_EINDEX (likewise)
 * if pack_gather_batch met a sample index outside the dataset. */
pack_status pack_read_loss(pack_t* p, float* host_dst);

/* free's checkpoint (Section 2.2): the member's current fp32 weights in the blob layout. */
pack_status pack_read_weights(pack_t* p, int32_t k, float* host_dst, size_t n_floats);

/* argmax over classes of the last step's logits of member k (lowest index on ties).
 * host_dst: int32 [b_k]. */
pack_status pack_read_pred(pack_t* p, int32_t k, int32_t* host_dst);

/* Test hook: the gradients the last step applied to member k, in the blob layout.  A pack whose
 * members all use PACK_OPT_SGD applies W <- W - lr dW inside the kernels that produce dW and does not
 * store the gradient at all (that saves a write and a read of every parameter per step); such a pack
 * returns PACK_EINVAL here unless pack_keep_grads(p, 1) was called, which makes the same kernels store
 * the gradient as well.  pack_keep_grads plans the pack again (member state is carried over). */
pack_status pack_read_grads(pack_t* p, int32_t k, float* host_dst, size_t n_floats);
pack_status pack_keep_grads(pack_t* p, int32_t on);

/* Test hook: the last step's logits of member k, row-major float [b_k, C_k]. */
pack_status pack_read_logits(pack_t* p, int32_t k, float* host_dst, size_t n_floats);

/* Number of floats in member k's blob; 0 if p is null or k is out of range. */
size_t pack_num_params(const pack_t* p, int32_t k);

/* Number of classes C_k of member k; 0 if out of range. */
int32_t pack_num_classes(const pack_t* p, int32_t k);

/* Number of kernel launches one pack_step enqueues (a packing figure of merit: K members cost
 * one launch sequence instead of K). */
int32_t pack_num_launches(const pack_t* p);

/* Bytes of device memory the pack holds (the paper's memory metric, Section 4.2: allocated). */
size_t pack_device_bytes(const pack_t* p);

/* Per-launch timing, for benchmarks: after pack_profile_start every `every`-th pack_step (the
 * first one included; every >= 1) brackets launch number `which` of its sequence (all launches
 * if which < 0) with a pair of events on the pack's stream.  An event costs a few microseconds
 * of stream time, which is why a long timed run samples its steps.  pack_profile_stop waits for the stream, writes the summed milliseconds and the
 * number of samples per launch index into ms_sum / count (host, pack_num_launches entries
 * each) and switches timing off.  pack_launch_name writes the kernel family of launch i
 * ("gemm_lin_fwd", "sgd_update", ...) into buf (host, n bytes, always terminated).
 * Errors: PACK_EINVAL (null, index out of range), PACK_EDEVICE. */
pack_status pack_profile_start(pack_t* p, int32_t which, int32_t every);
pack_status pack_profile_stop(pack_t* p, float* ms_sum, int32_t* count);
pack_status pack_launch_name(const pack_t* p, int32_t i, char* buf, size_t n);

/* Multiply-add work of launch i: 2 * rows * columns * reduction summed over the matrix products
 * the launch executes (0 for launches that are not matrix products).  flops: host. */
pack_status pack_launch_flops(const pack_t* p, int32_t i, double* flops);

/* Algorithmic bytes of launch i if it is a matrix-product launch: every operand read once (an operand
 * that several members share, the input batch of Section 3.4 or its im2col copy, once for the whole
 * launch), every result written once, plus, where the update is applied in the same kernel, the
 * weights read and written and their bf16 copy written (0 for other launches).  bytes: host. */
pack_status pack_launch_bytes(const pack_t* p, int32_t i, double* bytes);

/* Tile shape of launch i, for tests and measurements that need to know which kernel form the planner
 * chose: rows and columns of an output tile, and lean != 0 for the forms that keep one operand buffer and
 * one register stage (more workgroups per compute unit).  All three are 0 for launches that are not
 * matrix products.  The choice never changes results.  Outputs: host int32. */
pack_status pack_launch_tile(const pack_t* p, int32_t i, int32_t* tile_rows, int32_t* tile_cols, int32_t* lean);

/* Thread-local text describing the last failing call on this thread ("" if none). */
const char* pack_last_error(void);

/* free (Section 2.2): waits for the stream and releases everything the pack owns.  Null is a no-op. */
void pack_destroy(pack_t* p);

#ifdef __cplusplus
}
#endif
#endif /* PACK_H */
