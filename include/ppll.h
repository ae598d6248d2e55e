/*
 * ppll.h -- C ABI of libppll.so: one gradient-isolated block's local training
 * step on one MI355X (gfx950), and a single-GPU pipeline of K such blocks.
 *
 * Method (paper: Section 3.2 and Algorithm 1).  A network is cut into K
 * modules M_1..M_K, each with its own auxiliary network A_j and optimizer.
 * Process P_j repeats: take (x_{j-1}, y) from the buffer before it; forward
 * x_j = M_j(x_{j-1}); put (x_j, y) into the buffer after it; compute the
 * gradient of the local loss w.r.t. (theta_j, gamma_j) only -- nothing flows
 * into x_{j-1} (Sections 3.1-3.2, gradient isolation); update.  One
 * ppll_block_step is one pass of that loop body for one j; ppll_pipeline_step
 * feeds one batch to K blocks linked by bounded FIFO buffers of (x_j, y).
 *
 * Conventions common to all calls
 *  - Every function returns an int status (PPLL_OK = 0).  Nothing throws,
 *    aborts or exits.  ppll_last_error() gives the text of the calling thread's
 *    last failure.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device;
 *    "host" pointers are ordinary host memory.  All device pointers must be
 *    16-byte aligned.
 *  - The caller allocates and frees every device byte (workspace, inputs,
 *    outputs, loss) and owns the HIP streams.  The library carves parameters,
 *    optimizer moments, saved activations and queue slots out of the workspace
 *    and owns only its host-side records, events and side streams.
 *  - Argument errors are detected on the host before anything is enqueued and
 *    leave the handle untouched.  An out-of-range label raises a sticky device
 *    flag that the next *_sync reports as PPLL_ERR_LABEL.
 *  - Layouts: images NHWC [B,H,W,C]; tokens [B,T,D] row-major; ResNet
 *    activations NHWC [B,H,W,C]; weight matrices [in,out] row-major; 3x3
 *    filters [ky,kx,Cin,Cout].  Activations are fp32 on the PPLL_FP32 path and
 *    bf16 on the PPLL_BF16 path; labels are int32 in [0, num_classes).
 *  - A handle is used by one host thread at a time.
 */
#ifndef PPLL_H_
#define PPLL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PPLL_OK = 0,
  PPLL_ERR_NULL = 1,      /* a required pointer is null                          */
  PPLL_ERR_CONFIG = 2,    /* configuration outside what the kernels support      */
  PPLL_ERR_SHAPE = 3,     /* size/count argument does not match the config       */
  PPLL_ERR_WORKSPACE = 4, /* workspace too small or misaligned                   */
  PPLL_ERR_HIP = 5,       /* a HIP runtime call failed                           */
  PPLL_ERR_LABEL = 6,     /* a label was outside [0, num_classes)                */
  PPLL_ERR_STATE = 7      /* handle destroyed / call out of order                */
};

enum { PPLL_VIT = 0, PPLL_RESNET = 1 };
enum { PPLL_FP32 = 0, PPLL_BF16 = 1 };
enum { PPLL_IN_IMAGE = 0, PPLL_IN_ACTIVATION = 1 };
enum { PPLL_SGD = 0, PPLL_ADAMW = 1 };
/* tensor kinds for ppll_block_read_tensor / write_tensor */
enum { PPLL_T_PARAM = 0, PPLL_T_GRAD = 1, PPLL_T_MOMENT1 = 2, PPLL_T_MOMENT2 = 3,
       PPLL_T_BN_MEAN = 4, PPLL_T_BN_VAR = 5 };

/* Shape and hyper-parameters of one block = module M_j + auxiliary net A_j
 * (Section 3.2; model families and optimizer of Sections 4.1-4.2).
 * ViT: [patch-embed + cls + pos if PPLL_IN_IMAGE] -> depth pre-LN encoder
 * layers -> x_out; aux = aux_depth encoder layers -> LayerNorm -> cls token ->
 * Linear(dim, num_classes).  ResNet: [stem conv3x3 (img_c -> input channels)-
 * BN-ReLU if PPLL_IN_IMAGE] -> n_basic_blocks x (conv3x3-BN-ReLU-conv3x3-BN,
 * + shortcut, ReLU) -> x_out [batch, height, width, channels]; aux = conv3x3
 * stride 2 (channels -> aux_channels) -> BN -> ReLU -> global average ->
 * Linear.  With transition_block = i+1 basic block i is the one of the CIFAR
 * ResNet (Section 4.1) that halves the map and doubles the channels: its first
 * convolution has stride 2, its shortcut takes every second pixel and appends
 * zero channels, the blocks before it work on [2*height, 2*width, channels/2]
 * and that is also the shape of x_in (of the stem's output with a stem). */
typedef struct {
  uint32_t struct_size;   /* = sizeof(ppll_block_config)                         */
  int32_t arch;           /* PPLL_VIT | PPLL_RESNET                              */
  int32_t precision;      /* PPLL_FP32 | PPLL_BF16 (fp32 master weights always)  */
  int32_t input_kind;     /* PPLL_IN_IMAGE (ViT patches, ResNet stem) | PPLL_IN_ACTIVATION */
  int32_t batch, num_classes;
  int32_t img_h, img_w, img_c, patch;                    /* ViT image input      */
  int32_t tokens, dim, heads, mlp_dim, depth, aux_depth; /* ViT                  */
  int32_t channels, height, width, n_basic_blocks, aux_channels; /* ResNet       */
  int32_t transition_block; /* ResNet: 0 = none, i+1 = basic block i downsamples */
  int32_t optimizer;      /* PPLL_SGD | PPLL_ADAMW                               */
  float momentum;         /* SGD                                                 */
  int32_t nesterov;       /* SGD                                                 */
  float weight_decay;     /* SGD: coupled L2; AdamW: decoupled                   */
  float beta1, beta2, adam_eps;
  float ln_eps, bn_eps, bn_momentum;
  uint64_t seed;          /* used only when no initial parameters are supplied   */
} ppll_block_config;

typedef struct ppll_block ppll_block_t;
typedef struct ppll_pipeline ppll_pipeline_t;

/* Text of the calling thread's most recent failure (static storage, never null). */
const char* ppll_last_error(void);

/* Host-only size queries.  workspace: device bytes ppll_block_init needs;
 * param: bytes of the flat fp32 parameter blob (theta_j then gamma_j, tensor
 * order as reported by ppll_block_tensor_info); in/out: bytes of x_in / x_out
 * in the path's activation type. */
int ppll_block_workspace_bytes(const ppll_block_config* cfg, size_t* bytes);
int ppll_block_param_bytes(const ppll_block_config* cfg, size_t* bytes);
int ppll_block_in_bytes(const ppll_block_config* cfg, size_t* bytes);
int ppll_block_out_bytes(const ppll_block_config* cfg, size_t* bytes);

/* Algorithm 1, initialisation line: create block j's parameters (theta_j,
 * gamma_j) and optimizer state inside `workspace_dev`.
 * init_params_host: flat fp32 blob of ppll_block_param_bytes bytes, or null for a
 * seeded draw (weights N(0, 0.02^2), conv N(0, 2/(9 Cin)), biases 0, norm
 * scales 1).  The copy is done when the call returns.  hip_stream: a
 * hipStream_t (null = default stream) used for the set-up work.  *out receives
 * the handle; the workspace must outlive it. */
int ppll_block_init(const ppll_block_config* cfg, void* workspace_dev, size_t workspace_bytes,
                    const float* init_params_host, void* hip_stream, ppll_block_t** out);

/* Algorithm 1, loop body for one module: forward x_out = M_j(x_in) with the
 * parameters as they are before this call's update (that is what the algorithm
 * pushes to the next buffer); auxiliary forward; mean softmax cross-entropy
 * against `labels`; backward through A_j and M_j, stopping at x_in; optimizer
 * update of every tensor with learning rate `lr`.
 * Asynchronous on `hip_stream`.  x_in_dev [in_bytes] and labels_dev [batch] are
 * read only; x_out_dev [out_bytes] is written during the forward part and read
 * again by the backward part, so all three must stay valid and unmodified until
 * the stream has passed this call's work.  loss_dev: one float on the device
 * (may be null; ppll_block_sync still returns the loss).
 * A block with wide layers also launches part of its backward pass (the weight
 * gradients of upper layers) on a stream of its own, created at first use at
 * the default priority, forked from and joined back into `hip_stream` inside
 * this call: everything the call enqueued is complete once `hip_stream` has
 * passed it, and a caller never sees that stream. */
int ppll_block_step(ppll_block_t* blk, const void* x_in_dev, const int32_t* labels_dev, float lr,
                    void* x_out_dev, float* loss_dev, void* hip_stream);

/* Evaluation-mode forward of the block (how the paper's accuracies, Section 4.4, are taken once
 * training has run): x_out = M_j(x_in) with BatchNorm normalising by its running statistics; no
 * loss, no gradients, no update, running statistics unchanged.  x_in_dev / x_out_dev as in
 * ppll_block_step.  If logits_dev is non-null the block's auxiliary network is applied to x_out as
 * well and its class scores, [batch, num_classes] fp32 (device memory, 16-byte aligned), are
 * written there: for the last block of a network these are the network's predictions.  Enqueued
 * on hip_stream; the block's activation scratch is overwritten, so it must not overlap a step of
 * the same block in flight on another stream. */
int ppll_block_forward_eval(ppll_block_t* block, const void* x_in_dev, void* x_out_dev, float* logits_dev,
                            void* hip_stream);

/* For callers that cannot allocate device memory or let a library do it (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it) and that have no spare block workspace to evaluate in:
 * ppll_block_forward_eval with every intermediate activation placed in a buffer that is part of the library's
 * own device image, PPLL_EVAL_SCRATCH_BYTES long, instead of the block's workspace.  The call allocates nothing
 * on host or device and creates no stream or event; it reads the block's parameters and running statistics and
 * writes only x_out_dev, logits_dev and that buffer, so the activations a training step of the same block has
 * saved stay intact.  Results are bit-identical to ppll_block_forward_eval.
 *  - Limit: all layers share one set of activation buffers; a block whose largest layer needs more than
 *    PPLL_EVAL_SCRATCH_BYTES (a ViT stage of width 384, MLP 1536, 65 tokens fits up to batch 74) is refused
 *    with PPLL_ERR_WORKSPACE before anything is enqueued.
 *  - Every GPU the library has been used on holds its own copy of the buffer until the process ends; its
 *    address is looked up once per device by ppll_block_init.  The block must live on the current device
 *    (PPLL_ERR_STATE otherwise).
 *  - All calls on one GPU share that GPU's buffer, whatever block or stream they are made for: calls that
 *    overlap in time on one GPU race.  Order them on one stream or with events.  Nothing in the buffer has to
 *    start at zero (every kernel of the path writes what it later reads), so it is never cleared and keeps the
 *    previous call's contents. */
#define PPLL_EVAL_SCRATCH_BYTES (64u << 20)
int ppll_block_forward_eval_noalloc(ppll_block_t* block, const void* x_in_dev, void* x_out_dev, float* logits_dev,
                                    void* hip_stream);

/* Waits for the stream of the last step; returns that step's loss in
 * *loss_host (nullable).  Reports PPLL_ERR_LABEL / PPLL_ERR_HIP raised since the
 * previous sync. */
int ppll_block_sync(ppll_block_t* blk, float* loss_host);

/* Parameter-table access, for parity checks and checkpointing.  index runs
 * over 0..count-1 of the kind: parameter tensors for PARAM/GRAD/MOMENT*, BN
 * layers for BN_MEAN/BN_VAR.  n must equal the tensor's element count.  These
 * calls synchronise the block's stream. */
int ppll_block_tensor_count(ppll_block_t* blk, int32_t kind, int32_t* count);
int ppll_block_tensor_info(ppll_block_t* blk, int32_t kind, int32_t index, const char** name, size_t* n);
int ppll_block_read_tensor(ppll_block_t* blk, int32_t kind, int32_t index, float* host_out, size_t n);
int ppll_block_write_tensor(ppll_block_t* blk, int32_t kind, int32_t index, const float* host_in, size_t n);

/* Ends the block: waits for its last stream, releases the events and the side stream it created, and marks the
 * handle destroyed.  Device memory belongs to the caller.  The small host-side record itself stays allocated for
 * the life of the process, so that a later call with the stale handle is reported as PPLL_ERR_STATE instead of
 * touching freed memory. */
int ppll_block_destroy(ppll_block_t* blk);

/* Pipeline of K blocks on K HIP streams of one GPU (Algorithm 1, "parallel
 * execution for all j", with the buffers B_j as device ring buffers of
 * `queue_depth` slots holding (x_j, y); blocking FIFO: every batch is consumed
 * once, in order, by every block, so the values equal sequential local
 * learning).  cfgs[j+1]'s input must have the shape of cfgs[j]'s output and
 * the same batch, precision and class count. */
int ppll_pipeline_workspace_bytes(const ppll_block_config* cfgs, int32_t K, int32_t queue_depth, size_t* bytes);
int ppll_pipeline_init(const ppll_block_config* cfgs, int32_t K, int32_t queue_depth,
                       void* workspace_dev, size_t workspace_bytes, void* const* hip_streams /*K*/,
                       const float* const* init_params_host /*K entries or null*/, ppll_pipeline_t** out);

/* Enqueue one batch: copies (x0, labels) into the input slot on stream 0, then
 * for j = 0..K-1 on stream j: wait until the slot before it is ready and the
 * slot after it is free, forward into that slot, signal it, then auxiliary
 * forward, loss, backward, update, and release the input slot.  Returns after
 * enqueueing.  x0_dev / labels_dev must stay unmodified until stream 0 has
 * passed the copy (ppll_pipeline_sync guarantees it).  losses_dev: K floats on
 * the device, nullable. */
int ppll_pipeline_step(ppll_pipeline_t* pipe, const void* x0_dev, const int32_t* labels_dev, float lr,
                       float* losses_dev);

/* Waits for all K streams; losses_host (nullable) receives the K local losses
 * of the last batch. */
int ppll_pipeline_sync(ppll_pipeline_t* pipe, float* losses_host);

/* Borrow block j's handle (valid until ppll_pipeline_destroy) for tensor access. */
int ppll_pipeline_block(ppll_pipeline_t* pipe, int32_t j, ppll_block_t** borrowed);

/* Device address and byte size of the last block's most recent output. */
int ppll_pipeline_output(ppll_pipeline_t* pipe, const void** x_out_dev, size_t* bytes);

/* Ends the pipeline and its K blocks (as ppll_block_destroy: handles are marked destroyed, their host-side
 * records stay allocated so that stale handles are reported, not dereferenced after free). */
int ppll_pipeline_destroy(ppll_pipeline_t* pipe);

/* Measurement aid (no part of the method), per block.  While it is on for a block, every launch of the bf16
 * matrix-core GEMM kernel (gemm_mfma_kernel, all variants) and of the bf16 matrix-core convolution kernel that the
 * block's steps make is bracketed by a pair of HIP events on its own stream (a split-K reduce that may follow is
 * outside the bracket), and the block keeps every launch on the step's own stream (no side stream for weight
 * gradients), so that each bracket holds one kernel running alone.  Other blocks are not affected.
 * ppll_block_profile_read waits for those events and returns, since the previous read: the summed duration of the
 * GEMM launches in milliseconds, their algorithmic flops 2*M*N*K, and their count (each pointer nullable);
 * products with fewer than 256 output rows (the class-token products of a pruned last auxiliary layer, Section
 * 3.2's auxiliary network) are kept apart and read with ppll_block_profile_read_small;
 * ppll_block_profile_read_conv the same for the convolution launches (forward and input gradient of the ResNet
 * blocks) with their algorithmic bytes: input tensor + output tensor + filter once each, plus the two tensors of
 * the fused shortcut gradient where present.  The events add host and stream overhead: time whole steps with it off. */
int ppll_block_profile_enable(ppll_block_t* block, int32_t on);
int ppll_block_profile_read(ppll_block_t* block, double* gemm_ms, double* gemm_flops, int64_t* gemm_launches);
int ppll_block_profile_read_conv(ppll_block_t* block, double* conv_ms, double* conv_bytes, int64_t* conv_launches);
int ppll_block_profile_read_small(ppll_block_t* block, double* gemm_ms, double* gemm_flops, int64_t* gemm_launches);

/* Phase timers in the symbols of the paper's time model (Section 3.3: S_PPLL = f_1 + f_a1 + B_a1 +
 * U_a1): with timers on, every step of the block records HIP events on its stream at the ends of
 * the module forward (f), the auxiliary forward with the local loss (f_a), the backward through
 * auxiliary network and module including all parameter gradients (B), and the update (U).
 * ppll_block_phase_times waits for the block's last step and writes its four durations in
 * milliseconds to ms[0..3] (host memory) in that order; PPLL_ERR_STATE if timers are off or no step
 * has run.  The events cost a little host time per step: leave timers off when timing whole steps. */
int ppll_block_phase_timers(ppll_block_t* block, int32_t on);
int ppll_block_phase_times(ppll_block_t* block, float* ms);

/* Measurement aid: one plain copy kernel (copy_probe_kernel) moving `bytes` (a multiple of 16)
 * from src_dev to dst_dev on `hip_stream`.  Its known traffic (bytes read, bytes written) is
 * what the hardware byte counters of a profiler run are scaled against. */
int ppll_probe_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PPLL_H_ */
