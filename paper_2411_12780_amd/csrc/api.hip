// C ABI of libppll.so (see include/ppll.h): argument checks on the host, then
// the block engine / the K-stream pipeline.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "block.h"

namespace ppll {
static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}
}  // namespace ppll

using namespace ppll;

struct ppll_block {
  Block b;
};

// Activation scratch of ppll_block_forward_eval_noalloc: part of the library's device image, so every GPU the
// library runs on holds its own copy, at its own address, until the process ends.  In host code the name below
// is only a handle for hipGetSymbolAddress; the address kernels can use is looked up once per device
// (scratch_lookup) and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[PPLL_EVAL_SCRATCH_BYTES];

struct ppll_pipeline {
  int K = 0, depth = 0;
  bool alive = true;
  std::vector<ppll_block*> blocks;
  std::vector<hipStream_t> streams;
  // slot storage: in_slots[d] holds a copy of (x0, y); q[j][d] holds (x_{j+1}, y) for j < K-1
  std::vector<void*> in_x;
  std::vector<int32_t*> in_y;
  std::vector<std::vector<void*>> q_x;
  std::vector<std::vector<int32_t*>> q_y;
  void* last_out = nullptr;
  float* losses = nullptr;          // [K] device
  std::vector<std::vector<hipEvent_t>> ready, freed;   // [K-1][depth]
  std::vector<std::vector<char>> freed_set;
  long t = 0;
};

namespace {
// splitmix64 + Box-Muller: the seeded draw used when no parameters are supplied
struct Rng {
  uint64_t s;
  uint64_t next() {
    uint64_t z = (s += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
  }
  double uniform() { return ((next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
  double normal() { return std::sqrt(-2.0 * std::log(uniform())) * std::cos(6.283185307179586 * uniform()); }
};

bool ends_with(const std::string& s, const char* suf) {
  size_t n = strlen(suf);
  return s.size() >= n && s.compare(s.size() - n, n, suf) == 0;
}

void seeded_params(const Block& b, std::vector<float>& out) {
  Rng rng{b.cfg.seed * 0x2545F4914F6CDD1Dull + 1};
  out.assign(b.P, 0.f);
  for (const TensorDesc& t : b.tensors) {
    bool norm = t.name.find(".ln") != std::string::npos || t.name.find(".bn") != std::string::npos;
    bool conv = t.name.find("conv") != std::string::npos;
    double sd = 0.0, mean = 0.0;
    if (conv) sd = std::sqrt(2.0 / (double)t.rows);          // rows = 9 * Cin
    else if (norm && ends_with(t.name, ".g")) mean = 1.0;
    else if (ends_with(t.name, ".b")) sd = 0.0;
    else sd = 0.02;
    for (size_t i = 0; i < t.n; ++i) out[t.off + i] = (float)(mean + (sd > 0 ? sd * rng.normal() : 0.0));
  }
}

int check_aligned(const void* p, const char* what) {
  if (!p) { set_error("%s is null", what); return PPLL_ERR_NULL; }
  if (((uintptr_t)p) & 15) { set_error("%s is not 16-byte aligned", what); return PPLL_ERR_WORKSPACE; }
  return PPLL_OK;
}

int tensor_lookup(ppll_block* h, int32_t kind, int32_t index, float** dev, size_t* n, const char** name) {
  Block& b = h->b;
  if (kind == PPLL_T_BN_MEAN || kind == PPLL_T_BN_VAR) {
    if (index < 0 || index >= (int)b.bn_names.size()) { set_error("BN index %d out of range", index); return PPLL_ERR_SHAPE; }
    *dev = (kind == PPLL_T_BN_MEAN ? b.bn_mean_run : b.bn_var_run) + b.bn_off[index];
    *n = (size_t)b.bn_channels[index];
    if (name) *name = b.bn_names[index].c_str();
    return PPLL_OK;
  }
  if (index < 0 || index >= (int)b.tensors.size()) { set_error("tensor index %d out of range", index); return PPLL_ERR_SHAPE; }
  float* base = nullptr;
  switch (kind) {
    case PPLL_T_PARAM: base = b.params; break;
    case PPLL_T_GRAD: base = b.grads; break;
    case PPLL_T_MOMENT1: base = b.mom1; break;
    case PPLL_T_MOMENT2: base = b.mom2; break;
    default: set_error("unknown tensor kind %d", kind); return PPLL_ERR_SHAPE;
  }
  if (!base) { set_error("tensor kind %d does not exist for this optimizer", kind); return PPLL_ERR_STATE; }
  *dev = base + b.tensors[index].off;
  *n = b.tensors[index].n;
  if (name) *name = b.tensors[index].name.c_str();
  return PPLL_OK;
}

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each HIP device, null until looked up
std::mutex g_scratch_mu;

// Device address of the built-in scratch buffer on the current device; the first call on a device asks the runtime
// for it (with that device current, as it is here).  *dev_out receives the device ordinal.
int scratch_lookup(void** ptr_out, int* dev_out) {
  int dev = -1;
  PPLL_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_error("HIP device %d outside 0..%d", dev, kMaxDevices - 1); return PPLL_ERR_STATE; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_error("hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
      return PPLL_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  if (ptr_out) *ptr_out = g_scratch_ptr[dev];
  if (dev_out) *dev_out = dev;
  return PPLL_OK;
}

int block_alive(ppll_block* h) {
  if (!h) { set_error("block handle is null"); return PPLL_ERR_NULL; }
  if (!h->b.alive) { set_error("block handle was destroyed"); return PPLL_ERR_STATE; }
  return PPLL_OK;
}
}  // namespace

extern "C" {

const char* ppll_last_error(void) { return g_err; }

int ppll_probe_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream) {
  if (!src_dev || !dst_dev) { set_error("probe buffers are null"); return PPLL_ERR_NULL; }
  if ((((uintptr_t)src_dev) | ((uintptr_t)dst_dev) | bytes) & 15) { set_error("probe copy needs 16-byte alignment and size"); return PPLL_ERR_SHAPE; }
  return launch_copy_probe((hipStream_t)hip_stream, src_dev, dst_dev, bytes);
}

int ppll_block_workspace_bytes(const ppll_block_config* cfg, size_t* bytes) {
  PPLL_TRY(validate_config(cfg));
  if (!bytes) { set_error("bytes is null"); return PPLL_ERR_NULL; }
  Block b;
  b.cfg = *cfg;
  *bytes = b.plan(nullptr);
  return PPLL_OK;
}

int ppll_block_param_bytes(const ppll_block_config* cfg, size_t* bytes) {
  PPLL_TRY(validate_config(cfg));
  if (!bytes) { set_error("bytes is null"); return PPLL_ERR_NULL; }
  Block b;
  b.cfg = *cfg;
  b.plan(nullptr);
  *bytes = b.P * sizeof(float);
  return PPLL_OK;
}

int ppll_block_in_bytes(const ppll_block_config* cfg, size_t* bytes) {
  PPLL_TRY(validate_config(cfg));
  if (!bytes) { set_error("bytes is null"); return PPLL_ERR_NULL; }
  Block b;
  b.cfg = *cfg;
  *bytes = (size_t)b.in_elems() * dtype_size(cfg->precision == PPLL_BF16 ? BF16 : F32);
  return PPLL_OK;
}

int ppll_block_out_bytes(const ppll_block_config* cfg, size_t* bytes) {
  PPLL_TRY(validate_config(cfg));
  if (!bytes) { set_error("bytes is null"); return PPLL_ERR_NULL; }
  Block b;
  b.cfg = *cfg;
  *bytes = (size_t)b.out_elems() * dtype_size(cfg->precision == PPLL_BF16 ? BF16 : F32);
  return PPLL_OK;
}

int ppll_block_init(const ppll_block_config* cfg, void* workspace_dev, size_t workspace_bytes,
                    const float* init_params_host, void* hip_stream, ppll_block_t** out) {
  PPLL_TRY(validate_config(cfg));
  if (!out) { set_error("out is null"); return PPLL_ERR_NULL; }
  PPLL_TRY(check_aligned(workspace_dev, "workspace_dev"));
  int device = -1;
  PPLL_TRY(scratch_lookup(nullptr, &device));   // the library's set-up call: the built-in scratch address of this device
  ppll_block* h = new (std::nothrow) ppll_block();
  if (!h) { set_error("out of host memory"); return PPLL_ERR_STATE; }
  Block& b = h->b;
  b.cfg = *cfg;
  b.device = device;
  size_t need = b.plan((char*)workspace_dev);
  if (workspace_bytes < need) {
    set_error("workspace has %zu bytes, %zu needed", workspace_bytes, need);
    delete h;
    return PPLL_ERR_WORKSPACE;
  }
  b.ws = (char*)workspace_dev;
  b.ws_bytes = workspace_bytes;
  hipStream_t s = (hipStream_t)hip_stream;
  b.last_stream = s;
  std::vector<float> seeded;
  const float* src = init_params_host;
  if (!src) { seeded_params(b, seeded); src = seeded.data(); }
  auto fail = [&](int st) { delete h; return st; };
  auto hip_ok = [&](hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    set_error("%s failed: %s", what, hipGetErrorString(e));
    return false;
  };
  if (!hip_ok(hipMemcpyAsync(b.params, src, b.P * sizeof(float), hipMemcpyHostToDevice, s), "parameter upload")) return fail(PPLL_ERR_HIP);
  int st = launch_fill_zero(s, b.grads, b.P * sizeof(float));
  if (st == PPLL_OK && b.shadow) st = launch_refresh_shadow(s, b.params, b.shadow, b.P);
  if (st == PPLL_OK) st = launch_fill_zero(s, b.mom1, b.P * sizeof(float));
  if (st == PPLL_OK && b.mom2) st = launch_fill_zero(s, b.mom2, b.P * sizeof(float));
  if (st == PPLL_OK) st = launch_fill_zero(s, b.loss_dev, sizeof(float));
  if (st == PPLL_OK) st = launch_fill_zero(s, b.flag_dev, sizeof(int));
  if (st != PPLL_OK) return fail(st);
  size_t bn_total = 0;
  for (int c : b.bn_channels) bn_total += c;
  if (bn_total) {
    std::vector<float> ones(bn_total, 1.0f);
    if ((st = launch_fill_zero(s, b.bn_mean_run, bn_total * sizeof(float))) != PPLL_OK) return fail(st);
    if (!hip_ok(hipMemcpyAsync(b.bn_var_run, ones.data(), bn_total * sizeof(float), hipMemcpyHostToDevice, s), "BN state upload")) return fail(PPLL_ERR_HIP);
    if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return fail(PPLL_ERR_HIP);
  }
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return fail(PPLL_ERR_HIP);
  *out = h;
  return PPLL_OK;
}

int ppll_block_step(ppll_block_t* h, const void* x_in_dev, const int32_t* labels_dev, float lr, void* x_out_dev,
                    float* loss_dev, void* hip_stream) {
  PPLL_TRY(block_alive(h));
  PPLL_TRY(check_aligned(x_in_dev, "x_in_dev"));
  PPLL_TRY(check_aligned(x_out_dev, "x_out_dev"));
  if (!labels_dev) { set_error("labels_dev is null"); return PPLL_ERR_NULL; }
  if (!(lr == lr)) { set_error("lr is NaN"); return PPLL_ERR_CONFIG; }
  h->b.use_side = true;
  return h->b.step(x_in_dev, labels_dev, lr, x_out_dev, loss_dev, (hipStream_t)hip_stream, nullptr);
}

int ppll_block_forward_eval(ppll_block_t* h, const void* x_in_dev, void* x_out_dev, float* logits_dev, void* hip_stream) {
  PPLL_TRY(block_alive(h));
  PPLL_TRY(check_aligned(x_in_dev, "x_in_dev"));
  PPLL_TRY(check_aligned(x_out_dev, "x_out_dev"));
  if (logits_dev) PPLL_TRY(check_aligned(logits_dev, "logits_dev"));
  return h->b.forward_eval(x_in_dev, x_out_dev, logits_dev, (hipStream_t)hip_stream);
}

int ppll_block_forward_eval_noalloc(ppll_block_t* h, const void* x_in_dev, void* x_out_dev, float* logits_dev,
                                    void* hip_stream) {
  PPLL_TRY(block_alive(h));
  PPLL_TRY(check_aligned(x_in_dev, "x_in_dev"));
  PPLL_TRY(check_aligned(x_out_dev, "x_out_dev"));
  if (logits_dev) PPLL_TRY(check_aligned(logits_dev, "logits_dev"));
  int dev = -1;
  PPLL_HIP(hipGetDevice(&dev));
  if (dev != h->b.device) {
    set_error("the block lives on HIP device %d, the current device is %d", h->b.device, dev);
    return PPLL_ERR_STATE;
  }
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    ptr = g_scratch_ptr[dev];   // looked up by ppll_block_init on this device
  }
  if (!ptr) { set_error("the built-in scratch buffer of device %d was never looked up", dev); return PPLL_ERR_STATE; }
  return h->b.forward_eval_in_scratch(x_in_dev, x_out_dev, logits_dev, (hipStream_t)hip_stream, ptr,
                                      (size_t)PPLL_EVAL_SCRATCH_BYTES);
}

int ppll_block_sync(ppll_block_t* h, float* loss_host) {
  PPLL_TRY(block_alive(h));
  Block& b = h->b;
  PPLL_HIP(hipStreamSynchronize(b.last_stream));
  int flag = 0;
  PPLL_HIP(hipMemcpy(&flag, b.flag_dev, sizeof(int), hipMemcpyDeviceToHost));
  if (loss_host) PPLL_HIP(hipMemcpy(loss_host, b.loss_dev, sizeof(float), hipMemcpyDeviceToHost));
  if (flag) {
    int zero = 0;
    PPLL_HIP(hipMemcpy(b.flag_dev, &zero, sizeof(int), hipMemcpyHostToDevice));
    set_error("a label was outside [0, %d)", b.cfg.num_classes);
    return PPLL_ERR_LABEL;
  }
  return PPLL_OK;
}

int ppll_block_profile_enable(ppll_block_t* h, int32_t on) {
  PPLL_TRY(block_alive(h));
  h->b.time_launches = on != 0;
  return PPLL_OK;
}

namespace {
int profile_take(ppll_block* h, int kind, double* ms, double* units, int64_t* launches) {
  PPLL_TRY(block_alive(h));
  LaunchTimes& t = h->b.times;
  PPLL_TRY(profile_drain(t));
  if (ms) *ms = t.ms[kind];
  if (units) *units = t.units[kind];
  if (launches) *launches = t.launches[kind];
  t.ms[kind] = 0; t.units[kind] = 0; t.launches[kind] = 0;
  return PPLL_OK;
}
}  // namespace

int ppll_block_profile_read(ppll_block_t* h, double* gemm_ms, double* gemm_flops, int64_t* gemm_launches) {
  return profile_take(h, 0, gemm_ms, gemm_flops, gemm_launches);
}
int ppll_block_profile_read_conv(ppll_block_t* h, double* conv_ms, double* conv_bytes, int64_t* conv_launches) {
  return profile_take(h, 1, conv_ms, conv_bytes, conv_launches);
}
int ppll_block_profile_read_small(ppll_block_t* h, double* gemm_ms, double* gemm_flops, int64_t* gemm_launches) {
  return profile_take(h, 2, gemm_ms, gemm_flops, gemm_launches);
}

int ppll_block_phase_timers(ppll_block_t* h, int32_t on) {
  PPLL_TRY(block_alive(h));
  h->b.phase_timers = on != 0;
  if (!on)
    for (hipEvent_t& e : h->b.phase_ev) {
      if (e) (void)hipEventDestroy(e);
      e = nullptr;
    }
  return PPLL_OK;
}

int ppll_block_phase_times(ppll_block_t* h, float* ms) {
  PPLL_TRY(block_alive(h));
  if (!ms) { set_error("ms is null"); return PPLL_ERR_NULL; }
  Block& b = h->b;
  for (hipEvent_t e : b.phase_ev)
    if (!b.phase_timers || !e) { set_error("phase timers are off or no step has run with them"); return PPLL_ERR_STATE; }
  PPLL_HIP(hipEventSynchronize(b.phase_ev[4]));
  for (int i = 0; i < 4; ++i) PPLL_HIP(hipEventElapsedTime(&ms[i], b.phase_ev[i], b.phase_ev[i + 1]));
  return PPLL_OK;
}

int ppll_block_tensor_count(ppll_block_t* h, int32_t kind, int32_t* count) {
  PPLL_TRY(block_alive(h));
  if (!count) { set_error("count is null"); return PPLL_ERR_NULL; }
  if (kind == PPLL_T_BN_MEAN || kind == PPLL_T_BN_VAR) *count = (int32_t)h->b.bn_names.size();
  else if (kind >= PPLL_T_PARAM && kind <= PPLL_T_MOMENT2) *count = (int32_t)h->b.tensors.size();
  else { set_error("unknown tensor kind %d", kind); return PPLL_ERR_SHAPE; }
  return PPLL_OK;
}

int ppll_block_tensor_info(ppll_block_t* h, int32_t kind, int32_t index, const char** name, size_t* n) {
  PPLL_TRY(block_alive(h));
  float* dev; size_t cnt; const char* nm;
  PPLL_TRY(tensor_lookup(h, kind, index, &dev, &cnt, &nm));
  if (name) *name = nm;
  if (n) *n = cnt;
  return PPLL_OK;
}

int ppll_block_read_tensor(ppll_block_t* h, int32_t kind, int32_t index, float* host_out, size_t n) {
  PPLL_TRY(block_alive(h));
  if (!host_out) { set_error("host_out is null"); return PPLL_ERR_NULL; }
  float* dev; size_t cnt;
  PPLL_TRY(tensor_lookup(h, kind, index, &dev, &cnt, nullptr));
  if (n != cnt) { set_error("tensor has %zu elements, caller passed %zu", cnt, n); return PPLL_ERR_SHAPE; }
  PPLL_HIP(hipStreamSynchronize(h->b.last_stream));
  PPLL_HIP(hipMemcpy(host_out, dev, n * sizeof(float), hipMemcpyDeviceToHost));
  return PPLL_OK;
}

int ppll_block_write_tensor(ppll_block_t* h, int32_t kind, int32_t index, const float* host_in, size_t n) {
  PPLL_TRY(block_alive(h));
  if (!host_in) { set_error("host_in is null"); return PPLL_ERR_NULL; }
  float* dev; size_t cnt;
  PPLL_TRY(tensor_lookup(h, kind, index, &dev, &cnt, nullptr));
  if (n != cnt) { set_error("tensor has %zu elements, caller passed %zu", cnt, n); return PPLL_ERR_SHAPE; }
  PPLL_HIP(hipStreamSynchronize(h->b.last_stream));
  PPLL_HIP(hipMemcpy(dev, host_in, n * sizeof(float), hipMemcpyHostToDevice));
  if (kind == PPLL_T_PARAM && h->b.shadow) {
    size_t off = (size_t)(dev - h->b.params);
    PPLL_TRY(launch_refresh_shadow(h->b.last_stream, dev, h->b.shadow + off, n));
    PPLL_HIP(hipStreamSynchronize(h->b.last_stream));
  }
  return PPLL_OK;
}

int ppll_block_destroy(ppll_block_t* h) {
  if (!h) { set_error("block handle is null"); return PPLL_ERR_NULL; }
  if (!h->b.alive) { set_error("block handle was destroyed"); return PPLL_ERR_STATE; }
  (void)hipStreamSynchronize(h->b.last_stream);
  for (hipEvent_t& e : h->b.phase_ev) {
    if (e) (void)hipEventDestroy(e);
    e = nullptr;
  }
  h->b.side_destroy();
  profile_destroy(h->b.times);
  h->b.alive = false;   // the handle stays allocated so that later misuse is reported, not undefined
  return PPLL_OK;
}

// ------------------------------------------------------------------ pipeline
static int pipeline_check(const ppll_block_config* cfgs, int32_t K, int32_t depth) {
  if (!cfgs) { set_error("cfgs is null"); return PPLL_ERR_NULL; }
  if (K < 1 || K > 64) { set_error("K = %d outside 1..64", K); return PPLL_ERR_CONFIG; }
  if (depth < 1 || depth > 16) { set_error("queue_depth = %d outside 1..16", depth); return PPLL_ERR_CONFIG; }
  for (int j = 0; j < K; ++j) PPLL_TRY(validate_config(&cfgs[j]));
  for (int j = 1; j < K; ++j) {
    size_t a, b;
    ppll_block_out_bytes(&cfgs[j - 1], &a);
    ppll_block_in_bytes(&cfgs[j], &b);
    if (a != b || cfgs[j].batch != cfgs[0].batch || cfgs[j].precision != cfgs[0].precision ||
        cfgs[j].num_classes != cfgs[0].num_classes || cfgs[j].input_kind != PPLL_IN_ACTIVATION) {
      set_error("block %d does not accept block %d's output", j, j - 1);
      return PPLL_ERR_SHAPE;
    }
  }
  return PPLL_OK;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int ppll_pipeline_workspace_bytes(const ppll_block_config* cfgs, int32_t K, int32_t depth, size_t* bytes) {
  PPLL_TRY(pipeline_check(cfgs, K, depth));
  if (!bytes) { set_error("bytes is null"); return PPLL_ERR_NULL; }
  size_t total = 0, in_b, out_b, ws;
  const size_t lab = align256((size_t)cfgs[0].batch * sizeof(int32_t));
  ppll_block_in_bytes(&cfgs[0], &in_b);
  total += (size_t)depth * (align256(in_b) + lab);
  for (int j = 0; j < K; ++j) {
    ppll_block_workspace_bytes(&cfgs[j], &ws);
    ppll_block_out_bytes(&cfgs[j], &out_b);
    total += align256(ws);
    total += j < K - 1 ? (size_t)depth * (align256(out_b) + lab) : align256(out_b);
  }
  total += align256((size_t)K * sizeof(float));
  *bytes = total;
  return PPLL_OK;
}

int ppll_pipeline_init(const ppll_block_config* cfgs, int32_t K, int32_t depth, void* workspace_dev,
                       size_t workspace_bytes, void* const* hip_streams, const float* const* init_params_host,
                       ppll_pipeline_t** out) {
  size_t need;
  PPLL_TRY(ppll_pipeline_workspace_bytes(cfgs, K, depth, &need));
  if (!out) { set_error("out is null"); return PPLL_ERR_NULL; }
  if (!hip_streams) { set_error("hip_streams is null"); return PPLL_ERR_NULL; }
  PPLL_TRY(check_aligned(workspace_dev, "workspace_dev"));
  if (workspace_bytes < need) { set_error("workspace has %zu bytes, %zu needed", workspace_bytes, need); return PPLL_ERR_WORKSPACE; }
  ppll_pipeline* p = new (std::nothrow) ppll_pipeline();
  if (!p) { set_error("out of host memory"); return PPLL_ERR_STATE; }
  p->K = K; p->depth = depth;
  char* cur = (char*)workspace_dev;
  auto take = [&](size_t b) { char* r = cur; cur += align256(b); return (void*)r; };
  size_t in_b, out_b, ws;
  const size_t lab = (size_t)cfgs[0].batch * sizeof(int32_t);
  ppll_block_in_bytes(&cfgs[0], &in_b);
  for (int d = 0; d < depth; ++d) { p->in_x.push_back(take(in_b)); p->in_y.push_back((int32_t*)take(lab)); }
  p->q_x.resize(K > 1 ? K - 1 : 0); p->q_y.resize(K > 1 ? K - 1 : 0);
  int st = PPLL_OK;
  for (int j = 0; j < K && st == PPLL_OK; ++j) {
    ppll_block_workspace_bytes(&cfgs[j], &ws);
    ppll_block_out_bytes(&cfgs[j], &out_b);
    void* bws = take(ws);
    if (j < K - 1) {
      for (int d = 0; d < depth; ++d) { p->q_x[j].push_back(take(out_b)); p->q_y[j].push_back((int32_t*)take(lab)); }
    } else {
      p->last_out = take(out_b);
    }
    ppll_block* h = nullptr;
    st = ppll_block_init(&cfgs[j], bws, ws, init_params_host ? init_params_host[j] : nullptr, hip_streams[j], &h);
    if (st == PPLL_OK) { p->blocks.push_back(h); p->streams.push_back((hipStream_t)hip_streams[j]); }
  }
  p->losses = (float*)take((size_t)K * sizeof(float));
  auto cleanup = [&]() {
    for (auto& v : p->ready) for (hipEvent_t e : v) (void)hipEventDestroy(e);
    for (auto& v : p->freed) for (hipEvent_t e : v) (void)hipEventDestroy(e);
    for (ppll_block* h : p->blocks) delete h;
    delete p;
  };
  if (st != PPLL_OK) { cleanup(); return st; }
  p->ready.resize(K > 1 ? K - 1 : 0); p->freed.resize(K > 1 ? K - 1 : 0); p->freed_set.resize(K > 1 ? K - 1 : 0);
  for (int j = 0; j < K - 1; ++j) {
    p->freed_set[j].assign(depth, 0);
    for (int d = 0; d < depth; ++d) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess) {
        set_error("hipEventCreate failed");
        cleanup();
        return PPLL_ERR_HIP;
      }
      p->ready[j].push_back(a); p->freed[j].push_back(b);
    }
  }
  *out = p;
  return PPLL_OK;
}

static int pipeline_alive(ppll_pipeline* p) {
  if (!p) { set_error("pipeline handle is null"); return PPLL_ERR_NULL; }
  if (!p->alive) { set_error("pipeline handle was destroyed"); return PPLL_ERR_STATE; }
  return PPLL_OK;
}

int ppll_pipeline_step(ppll_pipeline_t* p, const void* x0_dev, const int32_t* labels_dev, float lr, float* losses_dev) {
  PPLL_TRY(pipeline_alive(p));
  PPLL_TRY(check_aligned(x0_dev, "x0_dev"));
  if (!labels_dev) { set_error("labels_dev is null"); return PPLL_ERR_NULL; }
  if (!(lr == lr)) { set_error("lr is NaN"); return PPLL_ERR_CONFIG; }
  const int K = p->K, slot = (int)(p->t % p->depth);
  const size_t lab = (size_t)p->blocks[0]->b.cfg.batch * sizeof(int32_t);
  size_t in_b;
  ppll_block_in_bytes(&p->blocks[0]->b.cfg, &in_b);
  // the stream of block 0 has already passed the step that last read this input slot
  PPLL_HIP(hipMemcpyAsync(p->in_x[slot], x0_dev, in_b, hipMemcpyDeviceToDevice, p->streams[0]));
  PPLL_HIP(hipMemcpyAsync(p->in_y[slot], labels_dev, lab, hipMemcpyDeviceToDevice, p->streams[0]));
  for (int j = 0; j < K; ++j) {
    hipStream_t s = p->streams[j];
    const void* x_in = j == 0 ? p->in_x[slot] : p->q_x[j - 1][slot];
    const int32_t* y_in = j == 0 ? p->in_y[slot] : p->q_y[j - 1][slot];
    void* x_out = j < K - 1 ? p->q_x[j][slot] : p->last_out;
    if (j > 0) PPLL_HIP(hipStreamWaitEvent(s, p->ready[j - 1][slot], 0));            // get from B_{j-1}
    if (j < K - 1 && p->freed_set[j][slot]) PPLL_HIP(hipStreamWaitEvent(s, p->freed[j][slot], 0));   // room in B_j
    auto publish = [&]() -> int {
      if (j < K - 1) {                                                                  // put (x_j, y) into B_j
        PPLL_HIP(hipMemcpyAsync(p->q_y[j][slot], y_in, lab, hipMemcpyDeviceToDevice, s));
        PPLL_HIP(hipEventRecord(p->ready[j][slot], s));
      }
      return PPLL_OK;
    };
    float* loss_j = losses_dev ? losses_dev + j : nullptr;
    p->blocks[j]->b.use_side = false;   // the other blocks' streams fill the chip
    PPLL_TRY(p->blocks[j]->b.step(x_in, y_in, lr, x_out, p->losses + j, s, publish));
    if (loss_j) PPLL_HIP(hipMemcpyAsync(loss_j, p->losses + j, sizeof(float), hipMemcpyDeviceToDevice, s));
    if (j > 0) {                                                                        // slot of B_{j-1} is free again
      PPLL_HIP(hipEventRecord(p->freed[j - 1][slot], s));
      p->freed_set[j - 1][slot] = 1;
    }
  }
  ++p->t;
  return PPLL_OK;
}

int ppll_pipeline_sync(ppll_pipeline_t* p, float* losses_host) {
  PPLL_TRY(pipeline_alive(p));
  int status = PPLL_OK;
  for (int j = 0; j < p->K; ++j) {
    int st = ppll_block_sync(p->blocks[j], losses_host ? losses_host + j : nullptr);
    if (st != PPLL_OK && status == PPLL_OK) status = st;
  }
  return status;
}

int ppll_pipeline_block(ppll_pipeline_t* p, int32_t j, ppll_block_t** borrowed) {
  PPLL_TRY(pipeline_alive(p));
  if (!borrowed) { set_error("borrowed is null"); return PPLL_ERR_NULL; }
  if (j < 0 || j >= p->K) { set_error("block index %d outside 0..%d", j, p->K - 1); return PPLL_ERR_SHAPE; }
  *borrowed = p->blocks[j];
  return PPLL_OK;
}

int ppll_pipeline_output(ppll_pipeline_t* p, const void** x_out_dev, size_t* bytes) {
  PPLL_TRY(pipeline_alive(p));
  if (x_out_dev) *x_out_dev = p->last_out;
  if (bytes) ppll_block_out_bytes(&p->blocks[p->K - 1]->b.cfg, bytes);
  return PPLL_OK;
}

int ppll_pipeline_destroy(ppll_pipeline_t* p) {
  if (!p) { set_error("pipeline handle is null"); return PPLL_ERR_NULL; }
  if (!p->alive) { set_error("pipeline handle was destroyed"); return PPLL_ERR_STATE; }
  for (hipStream_t s : p->streams) (void)hipStreamSynchronize(s);
  for (auto& v : p->ready) for (hipEvent_t e : v) (void)hipEventDestroy(e);
  for (auto& v : p->freed) for (hipEvent_t e : v) (void)hipEventDestroy(e);
  p->ready.clear(); p->freed.clear();
  for (ppll_block* h : p->blocks) h->b.alive = false;
  p->alive = false;
  return PPLL_OK;
}

}  // extern "C"
