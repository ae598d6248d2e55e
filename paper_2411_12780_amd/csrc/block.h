// Block engine: the static plan (parameter table, workspace layout) and the
// kernel sequence of one local-block step (Algorithm 1, loop body of P_j).
#pragma once

#include <functional>
#include <string>
#include <vector>

#include "common.h"

namespace ppll {

struct TensorDesc {
  std::string name;
  size_t off;        // element offset in the flat fp32 blob
  size_t n;          // elements
  int rows, cols;    // [in, out] for matrices, rows = 1 for vectors; conv: rows = 9*Cin, cols = Cout
};

struct EncoderParams {   // element offsets into the blob
  size_t ln1_g, ln1_b, qkv_w, qkv_b, proj_w, proj_b, ln2_g, ln2_b, fc1_w, fc1_b, fc2_w, fc2_b;
};
struct EncoderActs {     // saved by the forward for the backward (h: gelu' at the MLP pre-activation, gl: its gelu)
  void *u1, *qkv, *att, *x1, *u2, *h, *gl, *x2;
  float *mean1, *rstd1, *mean2, *rstd2, *lse;
};
// Compact buffers of the last auxiliary encoder layer, of which only the class-token row is computed behind the
// key / value projection ([B, .] instead of [B*T, .]; see Block::encoder_fwd_cls).
struct ClsActs {
  void *q, *att, *x1, *u2, *h, *gl, *x2;          // forward (h: gelu' at the MLP pre-activation, gl: its gelu)
  void *d_h, *d_u2, *d_x1, *d_att, *d_q;          // backward
  float *mean2, *rstd2, *prob;                     // prob [B, H, T]
};
struct BasicBlockParams { size_t conv1_w, bn1_g, bn1_b, conv2_w, bn2_g, bn2_b; };
// conv1 maps [Hin, Win, Ci] to [Ho, Wo, Co] with `stride`; everything after it in the block is [Ho, Wo, Co]
struct BasicBlockDims { int Ci, Co, stride, Hin, Win, Ho, Wo; };
struct BasicBlockActs {
  void *c1, *y1, *c2, *out;
  void *d1, *d2;   // gradients at the outputs of conv1 / conv2, kept until the grouped weight-gradient launch
  float *mean1, *rstd1, *mean2, *rstd2;
};

// Which buffers an evaluation-mode forward writes its intermediate activations to.  Either every layer has a
// set of its own (the block's training buffers: per_layer / per_block point at them), or all layers share one
// set and only the layer outputs alternate between two buffers (shared[l % 2]; the two sets differ in x2 / out).
struct EvalBuffers {
  const EncoderActs* per_layer = nullptr;
  EncoderActs shared_enc[2] = {};
  const EncoderActs& enc(int l) const { return per_layer ? per_layer[l] : shared_enc[l & 1]; }
  const BasicBlockActs* per_block = nullptr;
  BasicBlockActs shared_rb[2] = {};
  const BasicBlockActs& rb(int i) const { return per_block ? per_block[i] : shared_rb[i & 1]; }
  void *patches = nullptr, *embed_tmp = nullptr, *x0 = nullptr, *z = nullptr;          // ViT
  float *head_mean = nullptr, *head_rstd = nullptr;
  void *stem_c = nullptr, *stem_y = nullptr, *stem_xp = nullptr, *stem_wp = nullptr;   // ResNet
  void *shortcut = nullptr, *aux_c = nullptr, *aux_y = nullptr, *pooled = nullptr;
  float *stem_mean = nullptr, *stem_rstd = nullptr, *aux_mean = nullptr, *aux_rstd = nullptr;
};

struct Block {
  ppll_block_config cfg{};
  int dt = F32;              // activation element type
  size_t esz = 4;
  bool alive = true;

  std::vector<TensorDesc> tensors;
  std::vector<std::string> bn_names;
  std::vector<int> bn_channels;
  size_t P = 0;              // total parameters

  // workspace carve-up (device)
  char* ws = nullptr;
  size_t ws_bytes = 0;
  float *params = nullptr, *grads = nullptr, *mom1 = nullptr, *mom2 = nullptr;
  uint16_t* shadow = nullptr;   // bf16 copy of params that the contractions read (bf16 path only)
  // weight operand of a contraction: the bf16 shadow on the bf16 path, else the fp32 master
  const void* wptr(size_t off) const { return shadow ? (const void*)(shadow + off) : (const void*)(params + off); }
  int wdt() const { return shadow ? BF16 : F32; }
  float *bn_mean_run = nullptr, *bn_var_run = nullptr;   // [sum of BN channels]
  std::vector<size_t> bn_off;
  float* loss_dev = nullptr;
  int* flag_dev = nullptr;
  float* partials = nullptr;
  size_t partial_floats = 0;
  ReduceQueue rq;                 // second stages of the gradient reductions, run in one launch before the update
  size_t arena_floats = 0;
  float* splitk = nullptr;       // split-K partial sums of the weight-gradient GEMMs
  size_t splitk_floats = 0;

  // ViT
  size_t pe_w = 0, pe_b = 0, cls = 0, pos = 0, head_ln_g = 0, head_ln_b = 0, head_w = 0, head_b = 0;
  std::vector<EncoderParams> enc_p;       // depth + aux_depth
  std::vector<EncoderActs> enc_a;
  void *patches = nullptr, *x0 = nullptr, *embed_tmp = nullptr;
  void *z = nullptr, *dz = nullptr, *dcls = nullptr;
  // The last auxiliary layer feeds the head through its class-token row alone, so behind its key / value projection
  // only that row is computed (exact: no other row of that layer reaches the loss).  Off without auxiliary layers.
  bool prune_cls = false;
  ClsActs cls_a{};
  float *head_mean = nullptr, *head_rstd = nullptr, *logits = nullptr, *dlogits = nullptr;
  // Backward buffers.  Every layer keeps the gradients its four weight-gradient products read
  // (layer-output gradient, mid-layer gradient, d_h, d_qkv) until the end of the backward pass,
  // where all those products run as one grouped launch.  g_res[l+1] is the gradient with respect
  // to the output of layer l, g_res[0] the one with respect to the input of layer 0.
  std::vector<void*> g_res, g_mid, d_h, d_qkv;
  void* d_u = nullptr;
  std::vector<GemmArgs> wgrad_jobs;   // weight-gradient products recorded during the backward pass
  // Side stream of the backward pass (created at first use, default priority).  The weight-gradient products of a
  // layer are launched there once the layer's backward is enqueued, so they run next to the input-gradient chain of
  // the layers below, which never reads them; the step's stream waits for the side stream before the update.
  // Off for blocks driven by a pipeline: there the other blocks' streams already fill the chip.
  bool use_side = true;
  bool time_launches = false;          // bracket every contraction launch of this block's steps with events
  LaunchTimes times;
  hipStream_t side = nullptr;
  hipEvent_t side_fork = nullptr, side_join = nullptr;
  bool side_busy = false;              // something was launched on the side stream in this step
  int side_launch_wgrads(hipStream_t s);   // launches wgrad_jobs on the side stream behind everything enqueued on s
  int side_wait(hipStream_t s);            // s waits for the side stream's work of this step
  void side_destroy();

  // ResNet
  std::vector<BasicBlockParams> rb_p;
  std::vector<BasicBlockActs> rb_a;
  std::vector<BasicBlockDims> rb_d;
  int in_h = 0, in_w = 0, in_c = 0;      // activation the first basic block reads
  bool stem = false;                     // conv3x3 (img_c -> in_c) - BN - ReLU on the image in front of the blocks
  size_t stem_w = 0, stem_g = 0, stem_b = 0;
  void *stem_c = nullptr, *stem_y = nullptr, *shortcut = nullptr;
  // bf16 path: the image padded to 16 channels and the stem filter padded likewise, so that the stem runs on the
  // 16-channel matrix-core kernels (null: the stem runs on the generic kernels)
  void *stem_xp = nullptr, *stem_wp = nullptr;
  bool stem_pad = false;
  int stem_conv_fwd(const void* x_in, void* xp, void* wp, void* out, hipStream_t s, float* stat = nullptr,
                    int* stat_blocks = nullptr);
  float *stem_mean = nullptr, *stem_rstd = nullptr;
  int bn_base = 0;                       // index of rb0.bn1 among the BatchNorm layers (1 behind a stem)
  size_t aux_conv_w = 0, aux_bn_g = 0, aux_bn_b = 0;
  void *aux_c = nullptr, *aux_y = nullptr, *pooled = nullptr, *dpooled = nullptr, *d_aux = nullptr;
  float *aux_mean = nullptr, *aux_rstd = nullptr;
  void *r_gA = nullptr, *r_gB = nullptr, *r_t1 = nullptr;

  float* loss_copy = nullptr;    // caller's loss slot of the step in flight (may be null)
  // Phase timers (off by default): events at the boundaries of module forward, auxiliary forward +
  // loss, backward, update, recorded on the step's stream.
  bool phase_timers = false;
  hipEvent_t phase_ev[5] = {};
  int mark_phase(int i, hipStream_t s);
  // Evaluation-mode forward: x_out = M_j(x_in) (BatchNorm with running statistics); with logits_out the
  // auxiliary network's class scores [batch, num_classes] fp32 as well.  Changes no state but scratch.
  int forward_eval(const void* x_in, void* x_out, float* logits_out, hipStream_t s);
  // The same with every intermediate activation inside [scratch, scratch + scratch_bytes) instead of the block's
  // own buffers (all layers share one set there).  PPLL_ERR_WORKSPACE, before anything is enqueued, if the
  // shapes need more than scratch_bytes.  Allocates nothing on host or device.
  int forward_eval_in_scratch(const void* x_in, void* x_out, float* logits_out, hipStream_t s, void* scratch,
                              size_t scratch_bytes);
  int device = -1;               // HIP device the block was created on
  long steps = 0;
  hipStream_t last_stream = nullptr;


  // Builds the parameter table and assigns every workspace pointer relative to
  // `base` (null: only measure).  Returns the bytes needed.
  size_t plan(char* base);

  size_t in_elems() const;
  size_t out_elems() const;

  // Forward of the module into x_out; `after_forward` runs on the host right
  // after the forward kernels are enqueued (the pipeline publishes the slot
  // there), then auxiliary forward, loss, backward and update are enqueued.
  int step(const void* x_in, const int32_t* labels, float lr, void* x_out, float* loss_out, hipStream_t s,
           const std::function<int()>& after_forward);

 private:
  int vit_step(const void* x_in, const int32_t* labels, void* x_out, hipStream_t s,
               const std::function<int()>& after_forward);
  int resnet_step(const void* x_in, const int32_t* labels, void* x_out, hipStream_t s,
                  const std::function<int()>& after_forward);
  int encoder_fwd(int l, const EncoderActs& a, const void* x, void* x2_out, hipStream_t s);
  int forward_eval_with(const EvalBuffers& e, const void* x_in, void* x_out, float* logits_out, hipStream_t s);
  size_t plan_eval_scratch(char* base, EvalBuffers* e) const;
  int encoder_bwd(int l, const void* x, const void* g_in, void* g_tmp, void* g_out, bool need_dx, hipStream_t s);
  int encoder_fwd_cls(int l, const void* x, hipStream_t s);
  int encoder_bwd_cls(int l, const void* x, const void* d_x2, void* g_out, hipStream_t s);
  // dW[in, out] (row stride ldw) = X^T dY over K rows and db = column sums of dY; recorded for the grouped launch when
  // the matrix-core kernel can take it, else run at once.  x_ld / dy_ld: row strides of X [K, in] and dY [K, out].
  int wgrad_product(const void* xin, long x_ld, int in_dim, const void* dy, long dy_ld, int out_dim, int K, float* dW,
                    long ldw, float* db, hipStream_t s);
  int update(float lr, hipStream_t s);
};

int validate_config(const ppll_block_config* cfg);

}  // namespace ppll
