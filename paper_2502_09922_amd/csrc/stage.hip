// Stage runtime behind the C ABI of include/ls_stage.h: block table, event-gated loader,
// workspace carving and the per-layer launch sequence.  Host code only; every device step
// is a kernel launched through kernels.hpp.
#include "../../include/ls_stage.h"
#include "kernels.hpp"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

// Scratch of the entry point that allocates nothing (ls_stage_decode_static): the fp32
// partial tiles of the decode GEMMs that split K across workgroups.  Every GPU the library
// runs on holds its own copy of this array, at its own address, until the process ends.  In
// host code the name is only a handle for hipGetSymbolAddress; kernels get the address that
// call returned.
static __device__ __align__(256) unsigned char scratch[LS_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

// Address of `scratch` on each device, looked up once per device with that device current.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

hipError_t static_scratch_of_current_device(int* dev_out, void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *dev_out = dev;
  *ptr_out = g_scratch_ptr[dev];
  return hipSuccess;
}

ls_status fail(ls_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define LS_HIP(call)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) return fail(LS_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

ls::LaunchTiming& ls::launch_timing() {
  thread_local LaunchTiming t;
  return t;
}

// Lets the other host-side sources of the library set the message ls_last_error() returns.
void ls::set_last_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }
inline size_t isz(const ls_cfg* c) { return c->dtype == LS_DTYPE_F32 ? 4 : 2; }

bool cfg_ok(const ls_cfg* c) {
  if (!c) return false;
  if (c->abi_version != LS_ABI_VERSION || c->dtype > LS_DTYPE_BF16) return false;
  if (!c->n_layers_total || !c->hidden || !c->n_q_heads || !c->n_kv_heads || !c->head_dim || !c->ffn) return false;
  if (c->n_q_heads % c->n_kv_heads) return false;
  if ((c->head_dim & 1) || c->head_dim > 256) return false;
  if (!c->max_batch || !c->max_seq || c->max_tokens < c->max_batch) return false;
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return false;
  // 32-bit row*column products inside kernels stay in range
  if ((uint64_t)c->max_tokens > (1u << 30) || (uint64_t)c->max_seq > (1u << 24)) return false;
  return true;
}

// ---- packed block format ----------------------------------------------------------------
struct TensorSpan { size_t off, bytes; };

// Fills spans (if non-null) and returns the tensor count of block `layer`, 0 if invalid.
int block_tensors(const ls_cfg* c, int layer, TensorSpan* spans, size_t* total) {
  if (!cfg_ok(c)) return 0;
  const size_t e = isz(c), d = c->hidden, hd = c->head_dim, F = c->ffn, V = c->vocab;
  size_t elems[6];
  int n = 0;
  if (layer >= 0 && layer < (int)c->n_layers_total) {
    elems[n++] = d;
    elems[n++] = (size_t)(c->n_q_heads + 2 * c->n_kv_heads) * hd * d;
    elems[n++] = d * (size_t)c->n_q_heads * hd;
    elems[n++] = d;
    elems[n++] = 2 * F * d;
    elems[n++] = d * F;
  } else if (layer == LS_BLOCK_EMBED && V) {
    elems[n++] = V * d;
  } else if (layer == (int)c->n_layers_total && V) {
    elems[n++] = d;
    elems[n++] = V * d;
  } else {
    return 0;
  }
  size_t off = 0;
  for (int i = 0; i < n; ++i) {
    if (spans) spans[i] = {off, elems[i] * e};
    off = up(off + elems[i] * e);
  }
  if (total) *total = off;
  return n;
}

bool span_ok(const ls_cfg* c, int lo, int hi) {
  return cfg_ok(c) && lo >= 0 && lo < hi && hi <= (int)c->n_layers_total;
}

// ---- workspace carving ------------------------------------------------------------------
struct Carve {
  size_t cs, x, y, qkv, attn, h, logits, row_seq, row_pos, last_rows, next_tok, xb, xb2, ss_a, ss_b, splitk, splitk_bytes,
      attn_part, attn_part_bytes, total;
};

Carve carve(const ls_cfg* c, int lo, int hi) {
  Carve w{};
  const size_t e = isz(c), T = c->max_tokens, B = c->max_batch, d = c->hidden;
  const size_t qkv_cols = (size_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
  const bool last = c->vocab && hi == (int)c->n_layers_total;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = up(off + bytes); return o; };
  w.cs = take((size_t)c->max_seq * (c->head_dim / 2) * 2 * sizeof(float));
  w.x = take(T * d * sizeof(float));
  w.y = take(T * d * e);
  w.qkv = take(T * qkv_cols * e);
  w.attn = take(T * (size_t)c->n_q_heads * c->head_dim * e);
  w.h = take(T * (size_t)c->ffn * e);
  w.logits = take(last ? B * (size_t)c->vocab * sizeof(float) : 0);
  w.row_seq = take(T * sizeof(int32_t));
  w.row_pos = take(T * sizeof(int32_t));
  w.last_rows = take(B * sizeof(int32_t));
  w.next_tok = take(B * sizeof(int32_t));
  // decode-step fusion: bf16 copies of the residual rows and per-tile sums of squares
  w.xb = take(B * d * e);
  w.xb2 = take(B * d * e);
  w.ss_a = take(B * ((d + 15) / 16) * sizeof(float));
  w.ss_b = take(B * ((d + 15) / 16) * sizeof(float));
  {
    // split-K scratch of the decode GEMMs for 17..64 rows (bf16 only)
    size_t cols = qkv_cols > 2 * (size_t)c->ffn ? qkv_cols : 2 * (size_t)c->ffn;
    if (d > cols) cols = d;
    if (last && c->vocab > cols) cols = c->vocab;
    w.splitk_bytes = (c->dtype == LS_DTYPE_BF16 && B > 16) ? ls::gemm_scratch_bytes((int)B, cols) : 0;
    w.splitk = take(w.splitk_bytes);
  }
  // partial results of the grouped-query decode attention for contexts split over workgroups
  w.attn_part_bytes = c->dtype == LS_DTYPE_BF16
                          ? ls::attn_decode_gqa_scratch_bytes((int)B, (int)c->n_q_heads, (int)c->n_kv_heads, (int)c->max_seq)
                          : 0;
  w.attn_part = take(w.attn_part_bytes);
  (void)lo;
  w.total = off;
  return w;
}

enum BlockState { NOT_LOADED = 0, ENQUEUED = 1 };
constexpr int PROBE_CAP = 512;

struct Block {
  int layer;
  size_t off, bytes;
  int state;
  bool timed;  // copy_start / loaded bracket a copy made with profiling on
  hipEvent_t copy_start, loaded;
  // the host has seen `loaded` complete since the block was enqueued: the bytes are in HBM for
  // all work enqueued from now on, on any stream, and the gate needs no event wait any more
  bool landed;
};

// The gate: order stream `st` after the block's copy (nothing to enqueue once the copy is
// known to have completed).
inline hipError_t gate(Block& b, hipStream_t st) {
  if (b.landed) return hipSuccess;
  if (hipEventQuery(b.loaded) == hipSuccess) {
    b.landed = true;
    return hipSuccess;
  }
  (void)hipGetLastError();  // hipErrorNotReady from the query is not an error
  return hipStreamWaitEvent(st, b.loaded, 0);
}

}  // namespace

struct ls_stage {
  ls_cfg cfg;
  int lo, hi;
  bool first, last;
  char* slab;
  char* ws;
  Carve w;
  std::vector<Block> blocks;  // [embed?] layers lo..hi-1 [head?]
  int layer0;                 // index in blocks of layer lo
  int device;             // HIP device the stage was created on
  void* static_scratch;   // this device's copy of the library's static scratch array
  bool profiling;
  bool compute_timed;
  int origin_block;  // first block copied with profiling on since the last reset, or -1
  std::vector<hipEvent_t> comp_start, comp_end;
  hipEvent_t pass_start = nullptr, pass_end = nullptr;  // around a whole profiled prompt pass
  // kernel probe: event pairs around one operator of one layer, a ring of PROBE_CAP pairs
  int probe_op, probe_layer, probe_phase;
  size_t probe_count;
  std::vector<hipEvent_t> probe_a, probe_b;    // recorded around the launch(es)
  std::vector<hipEvent_t> probe_ka, probe_kb;  // stamped by the runtime with the kernel's own start / stop
  std::vector<char> probe_exact;               // slot holds a kernel-exact pair

  Block* find(int layer) {
    for (auto& b : blocks)
      if (b.layer == layer) return &b;
    return nullptr;
  }
  const Block* find(int layer) const { return const_cast<ls_stage*>(this)->find(layer); }
};

extern "C" {

const char* ls_last_error(void) { return g_err; }

size_t ls_block_bytes(const ls_cfg* cfg, int layer) {
  size_t total = 0;
  return block_tensors(cfg, layer, nullptr, &total) ? total : 0;
}

int ls_block_tensor_count(const ls_cfg* cfg, int layer) { return block_tensors(cfg, layer, nullptr, nullptr); }

ls_status ls_block_tensor(const ls_cfg* cfg, int layer, int index, size_t* offset, size_t* bytes) {
  TensorSpan sp[6];
  int n = block_tensors(cfg, layer, sp, nullptr);
  if (!n) return fail(LS_ERR_INVALID_ARG, "ls_block_tensor: invalid shape or block index %d", layer);
  if (index < 0 || index >= n || !offset || !bytes)
    return fail(LS_ERR_INVALID_ARG, "ls_block_tensor: tensor index %d outside [0,%d)", index, n);
  *offset = sp[index].off;
  *bytes = sp[index].bytes;
  return LS_OK;
}

size_t ls_stage_slab_bytes(const ls_cfg* cfg, int lo, int hi) {
  if (!span_ok(cfg, lo, hi)) return 0;
  size_t total = 0;
  if (cfg->vocab && lo == 0) total += ls_block_bytes(cfg, LS_BLOCK_EMBED);
  for (int l = lo; l < hi; ++l) total += ls_block_bytes(cfg, l);
  if (cfg->vocab && hi == (int)cfg->n_layers_total) total += ls_block_bytes(cfg, hi);
  return total;
}

size_t ls_stage_workspace_bytes(const ls_cfg* cfg, int lo, int hi) {
  return span_ok(cfg, lo, hi) ? carve(cfg, lo, hi).total : 0;
}

size_t ls_stage_kv_bytes(const ls_cfg* cfg, int lo, int hi) {
  if (!span_ok(cfg, lo, hi)) return 0;
  return (size_t)(hi - lo) * cfg->max_batch * cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * isz(cfg);
}

ls_status ls_stage_create(const ls_cfg* cfg, int lo, int hi, void* weight_slab, size_t slab_bytes,
                          void* workspace, size_t ws_bytes, ls_stage** out) {
  if (!out) return fail(LS_ERR_INVALID_ARG, "ls_stage_create: out is NULL");
  if (!cfg_ok(cfg)) return fail(LS_ERR_INVALID_ARG, "ls_stage_create: invalid ls_cfg");
  if (!span_ok(cfg, lo, hi)) return fail(LS_ERR_BLOCK_RANGE, "ls_stage_create: span [%d,%d) invalid", lo, hi);
  if (!weight_slab || !workspace) return fail(LS_ERR_INVALID_ARG, "ls_stage_create: NULL buffer");
  if (((uintptr_t)weight_slab | (uintptr_t)workspace) & (ALIGN - 1))
    return fail(LS_ERR_INVALID_ARG, "ls_stage_create: buffers must be 256-byte aligned");
  if (slab_bytes < ls_stage_slab_bytes(cfg, lo, hi)) return fail(LS_ERR_OOM, "ls_stage_create: weight slab too small");
  Carve w = carve(cfg, lo, hi);
  if (ws_bytes < w.total) return fail(LS_ERR_OOM, "ls_stage_create: workspace too small");

  int device = -1;
  void* static_scratch = nullptr;
  {
    hipError_t e = static_scratch_of_current_device(&device, &static_scratch);
    if (e != hipSuccess) return fail(LS_ERR_HIP, "ls_stage_create: address of the static scratch: %s", hipGetErrorString(e));
  }
  ls_stage* s = new (std::nothrow) ls_stage();
  if (!s) return fail(LS_ERR_OOM, "ls_stage_create: host allocation failed");
  s->device = device;
  s->static_scratch = static_scratch;
  s->cfg = *cfg;
  s->lo = lo;
  s->hi = hi;
  s->first = cfg->vocab && lo == 0;
  s->last = cfg->vocab && hi == (int)cfg->n_layers_total;
  s->slab = (char*)weight_slab;
  s->ws = (char*)workspace;
  s->w = w;
  s->profiling = false;
  s->compute_timed = false;
  s->origin_block = -1;
  s->probe_op = LS_OP_NONE;
  s->probe_layer = s->probe_phase = 0;
  s->probe_count = 0;

  size_t off = 0;
  auto add = [&](int layer) {
    Block b{};
    b.layer = layer;
    b.off = off;
    b.bytes = ls_block_bytes(cfg, layer);
    b.state = NOT_LOADED;
    off += b.bytes;
    s->blocks.push_back(b);
  };
  if (s->first) add(LS_BLOCK_EMBED);
  s->layer0 = (int)s->blocks.size();
  for (int l = lo; l < hi; ++l) add(l);
  if (s->last) add(hi);

  auto cleanup = [&]() {
    for (auto& b : s->blocks) {
      if (b.copy_start) (void)hipEventDestroy(b.copy_start);
      if (b.loaded) (void)hipEventDestroy(b.loaded);
    }
    for (auto e : s->comp_start) (void)hipEventDestroy(e);
    for (auto e : s->comp_end) (void)hipEventDestroy(e);
    for (auto e : s->probe_a) (void)hipEventDestroy(e);
    for (auto e : s->probe_b) (void)hipEventDestroy(e);
    for (auto e : s->probe_ka) (void)hipEventDestroy(e);
    for (auto e : s->probe_kb) (void)hipEventDestroy(e);
    if (s->pass_start) (void)hipEventDestroy(s->pass_start);
    if (s->pass_end) (void)hipEventDestroy(s->pass_end);
    delete s;
  };
  for (auto& b : s->blocks) {
    if (hipEventCreate(&b.copy_start) != hipSuccess || hipEventCreate(&b.loaded) != hipSuccess) {
      cleanup();
      return fail(LS_ERR_HIP, "ls_stage_create: hipEventCreate failed");
    }
  }
  for (int l = lo; l < hi; ++l) {
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
      if (a) (void)hipEventDestroy(a);
      cleanup();
      return fail(LS_ERR_HIP, "ls_stage_create: hipEventCreate failed");
    }
    s->comp_start.push_back(a);
    s->comp_end.push_back(b);
  }

  if (hipEventCreate(&s->pass_start) != hipSuccess || hipEventCreate(&s->pass_end) != hipSuccess) {
    cleanup();
    return fail(LS_ERR_HIP, "ls_stage_create: hipEventCreate failed");
  }

  // cos/sin of pos * base^(-2i/hd), evaluated in double and stored as fp32 pairs
  const int half = cfg->head_dim / 2;
  std::vector<float> cs((size_t)cfg->max_seq * half * 2);
  for (uint32_t p = 0; p < cfg->max_seq; ++p)
    for (int i = 0; i < half; ++i) {
      double a = (double)p * std::pow((double)cfg->rope_base, -2.0 * i / (double)cfg->head_dim);
      cs[((size_t)p * half + i) * 2] = (float)std::cos(a);
      cs[((size_t)p * half + i) * 2 + 1] = (float)std::sin(a);
    }
  hipError_t e = hipMemcpy(s->ws + w.cs, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    cleanup();
    return fail(LS_ERR_HIP, "ls_stage_create: table upload: %s", hipGetErrorString(e));
  }
  *out = s;
  return LS_OK;
}

void ls_stage_destroy(ls_stage* s) {
  if (!s) return;
  for (auto& b : s->blocks) {
    (void)hipEventDestroy(b.copy_start);
    (void)hipEventDestroy(b.loaded);
  }
  for (auto e : s->comp_start) (void)hipEventDestroy(e);
  for (auto e : s->comp_end) (void)hipEventDestroy(e);
  for (auto e : s->probe_a) (void)hipEventDestroy(e);
  for (auto e : s->probe_b) (void)hipEventDestroy(e);
  for (auto e : s->probe_ka) (void)hipEventDestroy(e);
  for (auto e : s->probe_kb) (void)hipEventDestroy(e);
  (void)hipEventDestroy(s->pass_start);
  (void)hipEventDestroy(s->pass_end);
  delete s;
}

ls_status ls_stage_info(const ls_stage* s, ls_cfg* cfg, int* lo, int* hi) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_info: NULL stage");
  if (cfg) *cfg = s->cfg;
  if (lo) *lo = s->lo;
  if (hi) *hi = s->hi;
  return LS_OK;
}

size_t ls_stage_block_bytes(const ls_stage* s, int layer) {
  if (!s) return 0;
  const Block* b = s->find(layer);
  return b ? b->bytes : 0;
}

void* ls_stage_block_device_ptr(const ls_stage* s, int layer) {
  if (!s) return nullptr;
  const Block* b = s->find(layer);
  return b ? (void*)(s->slab + b->off) : nullptr;
}

ls_status ls_stage_load_block(ls_stage* s, const void* host_ptr, int layer, void* hip_stream) {
  if (!s || !host_ptr) return fail(LS_ERR_INVALID_ARG, "ls_stage_load_block: NULL argument");
  Block* b = s->find(layer);
  if (!b) return fail(LS_ERR_BLOCK_RANGE, "ls_stage_load_block: block %d is not held by stage [%d,%d)", layer, s->lo, s->hi);
  if (b->state != NOT_LOADED) return fail(LS_ERR_ALREADY_LOADED, "ls_stage_load_block: block %d already enqueued", layer);
  hipStream_t st = (hipStream_t)hip_stream;
  b->timed = s->profiling;
  if (s->profiling) {
    LS_HIP(hipEventRecord(b->copy_start, st));
    if (s->origin_block < 0) s->origin_block = (int)(b - s->blocks.data());
  }
  LS_HIP(hipMemcpyAsync(s->slab + b->off, host_ptr, b->bytes, hipMemcpyHostToDevice, st));
  LS_HIP(hipEventRecord(b->loaded, st));
  b->state = ENQUEUED;
  b->landed = false;
  return LS_OK;
}

ls_status ls_stage_load_layers(ls_stage* s, const void* host_ptr, int first, int last, void* hip_stream) {
  if (!s || !host_ptr) return fail(LS_ERR_INVALID_ARG, "ls_stage_load_layers: NULL argument");
  if (first < s->lo || last >= s->hi || first > last)
    return fail(LS_ERR_BLOCK_RANGE, "ls_stage_load_layers: layers [%d,%d] outside stage [%d,%d)", first, last, s->lo, s->hi);
  Block* b0 = s->find(first);
  size_t bytes = 0;
  for (int l = first; l <= last; ++l) {
    Block* b = s->find(l);
    if (b->state != NOT_LOADED) return fail(LS_ERR_ALREADY_LOADED, "ls_stage_load_layers: block %d already enqueued", l);
    bytes += b->bytes;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  if (s->profiling) {
    for (int l = first; l <= last; ++l) LS_HIP(hipEventRecord(s->find(l)->copy_start, st));
    if (s->origin_block < 0) s->origin_block = (int)(b0 - s->blocks.data());
  }
  LS_HIP(hipMemcpyAsync(s->slab + b0->off, host_ptr, bytes, hipMemcpyHostToDevice, st));
  for (int l = first; l <= last; ++l) {
    Block* b = s->find(l);
    b->timed = s->profiling;
    LS_HIP(hipEventRecord(b->loaded, st));
    b->state = ENQUEUED;
    b->landed = false;
  }
  return LS_OK;
}

ls_status ls_stage_adopt_block(ls_stage* s, int layer, void* hip_stream) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_adopt_block: NULL stage");
  Block* b = s->find(layer);
  if (!b) return fail(LS_ERR_BLOCK_RANGE, "ls_stage_adopt_block: block %d is not held by stage [%d,%d)", layer, s->lo, s->hi);
  if (b->state != NOT_LOADED) return fail(LS_ERR_ALREADY_LOADED, "ls_stage_adopt_block: block %d already enqueued", layer);
  b->timed = false;
  LS_HIP(hipEventRecord(b->loaded, (hipStream_t)hip_stream));
  b->state = ENQUEUED;
  b->landed = false;
  return LS_OK;
}

ls_status ls_stage_reset_blocks(ls_stage* s) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_reset_blocks: NULL stage");
  for (auto& b : s->blocks) {
    b.state = NOT_LOADED;
    b.timed = false;
    b.landed = false;
  }
  s->origin_block = -1;
  return LS_OK;
}

ls_status ls_stage_set_profiling(ls_stage* s, int on) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_set_profiling: NULL stage");
  s->profiling = on != 0;
  if (!on) s->compute_timed = false;
  return LS_OK;
}

}  // extern "C"

// ---- the forward pass -------------------------------------------------------------------
namespace {

// `gsc`: where GEMM kernels that split K across workgroups put their partial tiles.
ls_status forward(ls_stage* s, bool prefill, const void* in, const int32_t* cu_dev, int batch, int rows, int max_len,
                  const ls_kv* kv, void* out, float* logits_out, hipStream_t st, const ls::GemmScratch& gsc) {
  using namespace ls;
  const ls_cfg& c = s->cfg;
  const uint32_t dt = c.dtype;
  const int d = c.hidden, hq = c.n_q_heads, hkv = c.n_kv_heads, hd = c.head_dim, F = c.ffn;
  const int qkv_cols = (hq + 2 * hkv) * hd;
  const size_t e = isz(&c);
  char* ws = s->ws;
  float* x = (float*)(ws + s->w.x);
  void* y = ws + s->w.y;
  void* qkv = ws + s->w.qkv;
  void* attn = ws + s->w.attn;
  void* hbuf = ws + s->w.h;
  const float* cs = (const float*)(ws + s->w.cs);
  int32_t* row_seq = (int32_t*)(ws + s->w.row_seq);
  int32_t* row_pos = (int32_t*)(ws + s->w.row_pos);
  int32_t* last_rows = (int32_t*)(ws + s->w.last_rows);
  const bool timed = s->profiling && prefill;
  const bool probing = s->probe_op != LS_OP_NONE && s->probe_phase == (prefill ? 0 : 1) && !s->probe_a.empty();

  // PROBE(op, launch): bracket the launch with an event pair if this (op, layer) is probed
#define PROBE(op, launch)                                                        \
  do {                                                                           \
    const bool on_ = probing && s->probe_op == (op) && s->probe_layer == b.layer; \
    const size_t slot_ = s->probe_count % PROBE_CAP;                             \
    if (on_) {                                                                   \
      LS_HIP(hipEventRecord(s->probe_a[slot_], st));                             \
      LaunchTiming& lt_ = launch_timing();                                       \
      lt_.start = s->probe_ka[slot_];                                            \
      lt_.stop = s->probe_kb[slot_];                                             \
      lt_.used = false;                                                          \
    }                                                                            \
    launch;                                                                      \
    if (on_) {                                                                   \
      LaunchTiming& lt_ = launch_timing();                                       \
      s->probe_exact[slot_] = lt_.used;                                          \
      lt_.start = lt_.stop = nullptr;                                            \
      LS_HIP(hipEventRecord(s->probe_b[slot_], st));                             \
      s->probe_count++;                                                          \
    }                                                                            \
  } while (0)
  const size_t kv_layer = (size_t)c.max_batch * hkv * c.max_seq * hd * e;

  // ---- decode step with the RMSNorms folded into the weight-streaming GEMMs
  const bool fused = !prefill && dt == BF16 && d % 16 == 0 &&
                     (attn_decode_supported(hq, hkv, hd) || attn_decode_gqa_supported(hq, hkv, hd)) &&
                     gemm_decode_fusable(rows, qkv_cols, d) && gemm_decode_fusable(rows, d, hq * hd) &&
                     gemm_decode_fusable(rows, F, d) && gemm_decode_fusable(rows, d, F);
  if (fused) {
    __bf16* xb = (__bf16*)(ws + s->w.xb);
    __bf16* xb2 = (__bf16*)(ws + s->w.xb2);
    float* ss_a = (float*)(ws + s->w.ss_a);
    float* ss_b = (float*)(ws + s->w.ss_b);
    const void* table = nullptr;
    if (s->first) {
      Block* eb = s->find(LS_BLOCK_EMBED);
      LS_HIP(gate(*eb, st));
      table = s->slab + eb->off;
    }
    const int n_layers = s->hi - s->lo;
    // The gain of a norm is applied where the bf16 copy of the residual rows is written: by
    // the prologue (first layer's attention norm), by the O projection (the same layer's FFN
    // norm) and by the down projection (the NEXT layer's attention norm -- so a layer's last
    // kernel is also ordered after the next layer's block).
    auto gain = [&](int li, int tensor) {
      const Block& b = s->blocks[s->layer0 + li];
      TensorSpan sp[6];
      block_tensors(&c, b.layer, sp, nullptr);
      return (const __bf16*)(s->slab + b.off + sp[tensor].off);
    };
    LS_HIP(gate(s->blocks[s->layer0], st));  // the gate of the first layer
    launch_decode_prologue(dt, table, in, kv->seq_lens, batch, c.max_seq, d, c.vocab, row_seq, row_pos, last_rows, x,
                           xb, ss_a, gain(0, 0), st);
    for (int li = 0; li < n_layers; ++li) {
      Block& b = s->blocks[s->layer0 + li];
      TensorSpan sp[6];
      block_tensors(&c, b.layer, sp, nullptr);
      const char* base = s->slab + b.off;
      LS_HIP(gate(b, st));  // the gate
      char* kc = (char*)kv->k + li * kv_layer;
      char* vc = (char*)kv->v + li * kv_layer;
      const bool more = li + 1 < n_layers;
      SkinnyFusion f_qkv, f_o, f_gu, f_dn;
      f_qkv.ss_in = ss_a; f_qkv.n_part = d / 16; f_qkv.eps = c.rms_eps;
      f_o.xb_out = xb2; f_o.ss_out = ss_b; f_o.gamma_out = gain(li, 3);
      f_gu.ss_in = ss_b; f_gu.n_part = d / 16; f_gu.eps = c.rms_eps;
      // the last layer of a middle stage writes the stage output directly (no gain)
      f_dn.xb_out = (!more && !s->last) ? (__bf16*)out : xb; f_dn.ss_out = ss_a;
      f_dn.gamma_out = more ? gain(li + 1, 0) : nullptr;
      PROBE(LS_OP_GEMM_QKV, launch_gemm(dt, EPI_STORE, xb, base + sp[1].off, rows, qkv_cols, d, qkv, nullptr, st, &gsc, &f_qkv));
      PROBE(LS_OP_ATTENTION, launch_attention_block(dt, nullptr, batch, max_len, qkv, cs, kc, vc, row_seq, row_pos, rows,
                                                    hq, hkv, hd, c.max_seq, attn, st,
                                                    s->w.attn_part_bytes ? (float*)(ws + s->w.attn_part) : nullptr,
                                                    s->w.attn_part_bytes));
      PROBE(LS_OP_GEMM_O, launch_gemm(dt, EPI_RESID, attn, base + sp[2].off, rows, d, hq * hd, nullptr, x, st, &gsc, &f_o));
      PROBE(LS_OP_GEMM_GATEUP, launch_gemm(dt, EPI_SWIGLU, xb2, base + sp[4].off, rows, F, d, hbuf, nullptr, st, &gsc, &f_gu));
      if (more) LS_HIP(gate(s->blocks[s->layer0 + li + 1], st));  // its gain is read next
      PROBE(LS_OP_GEMM_DOWN, launch_gemm(dt, EPI_RESID, hbuf, base + sp[5].off, rows, d, F, nullptr, x, st, &gsc, &f_dn));
    }
    if (s->last) {
      Block* hb = s->find(s->hi);
      TensorSpan sp[6];
      block_tensors(&c, hb->layer, sp, nullptr);
      const char* base = s->slab + hb->off;
      LS_HIP(gate(*hb, st));
      float* logits = logits_out ? logits_out : (float*)(ws + s->w.logits);
      launch_rmsnorm(dt, x, base + sp[0].off, y, batch, d, c.rms_eps, last_rows, st);
      launch_gemm(dt, EPI_F32, y, base + sp[1].off, batch, c.vocab, d, logits, nullptr, st, &gsc);
      launch_argmax(logits, batch, c.vocab, (int32_t*)out, st);
    }
    LS_HIP(hipGetLastError());
    return LS_OK;
  }

  if (timed) LS_HIP(hipEventRecord(s->pass_start, st));
  if (prefill) launch_row_index_prefill(cu_dev, batch, rows, row_seq, row_pos, last_rows, st);
  else launch_row_index_decode(kv->seq_lens, batch, c.max_seq, row_seq, row_pos, last_rows, st);

  if (s->first) {
    Block* eb = s->find(LS_BLOCK_EMBED);
    LS_HIP(gate(*eb, st));  // gate: embedding block has landed
    launch_embed(dt, s->slab + eb->off, (const int32_t*)in, x, rows, d, c.vocab, st);
  } else {
    launch_load_hidden(dt, in, x, (size_t)rows * d, st);
  }

  for (int li = 0; li < s->hi - s->lo; ++li) {
    Block& b = s->blocks[s->layer0 + li];
    TensorSpan sp[6];
    block_tensors(&c, b.layer, sp, nullptr);
    const char* base = s->slab + b.off;
    // the gate: nothing of this layer may read its weights before its block has landed
    LS_HIP(gate(b, st));
    if (timed) LS_HIP(hipEventRecord(s->comp_start[li], st));
    char* kc = (char*)kv->k + li * kv_layer;
    char* vc = (char*)kv->v + li * kv_layer;

    PROBE(LS_OP_NORM, launch_rmsnorm(dt, x, base + sp[0].off, y, rows, d, c.rms_eps, nullptr, st));
    // many-row prompt passes: RoPE and the cache append ride in the QKV projection's epilogue
    const bool rope_in_gemm = prefill && dt == BF16 && rows > 64 && attn_prefill_supported(hq, hkv, hd) &&
                              gemm_mfma_rope_supported(rows, qkv_cols, d, hq, hkv, hd);
    if (rope_in_gemm) {
      RopeAppend ra;
      ra.cs = cs; ra.row_seq = row_seq; ra.row_pos = row_pos;
      ra.hq = hq; ra.hkv = hkv; ra.hd = hd; ra.max_seq = c.max_seq;
      ra.kc = (__bf16*)kc; ra.vc = (__bf16*)vc;
      PROBE(LS_OP_GEMM_QKV, launch_gemm_mfma_rope(y, base + sp[1].off, rows, qkv_cols, d, qkv, ra, st));
    } else {
      PROBE(LS_OP_GEMM_QKV, launch_gemm(dt, EPI_STORE, y, base + sp[1].off, rows, qkv_cols, d, qkv, nullptr, st, &gsc));
    }
    PROBE(LS_OP_ATTENTION, launch_attention_block(dt, cu_dev, batch, max_len, qkv, cs, kc, vc, row_seq, row_pos, rows,
                                                  hq, hkv, hd, c.max_seq, attn, st, nullptr, 0, rope_in_gemm));
    PROBE(LS_OP_GEMM_O, launch_gemm(dt, EPI_RESID, attn, base + sp[2].off, rows, d, hq * hd, nullptr, x, st, &gsc));
    launch_rmsnorm(dt, x, base + sp[3].off, y, rows, d, c.rms_eps, nullptr, st);
    PROBE(LS_OP_GEMM_GATEUP, launch_gemm(dt, EPI_SWIGLU, y, base + sp[4].off, rows, F, d, hbuf, nullptr, st, &gsc));
    PROBE(LS_OP_GEMM_DOWN, launch_gemm(dt, EPI_RESID, hbuf, base + sp[5].off, rows, d, F, nullptr, x, st, &gsc));
    if (timed) LS_HIP(hipEventRecord(s->comp_end[li], st));
  }
#undef PROBE
  if (timed) s->compute_timed = true;

  if (s->last) {
    Block* hb = s->find(s->hi);
    TensorSpan sp[6];
    block_tensors(&c, hb->layer, sp, nullptr);
    const char* base = s->slab + hb->off;
    LS_HIP(gate(*hb, st));  // gate: head block has landed
    float* logits = logits_out ? logits_out : (float*)(ws + s->w.logits);
    launch_rmsnorm(dt, x, base + sp[0].off, y, batch, d, c.rms_eps, last_rows, st);
    launch_gemm(dt, EPI_F32, y, base + sp[1].off, batch, c.vocab, d, logits, nullptr, st, &gsc);
    launch_argmax(logits, batch, c.vocab, (int32_t*)out, st);
  } else {
    launch_store_hidden(dt, x, out, (size_t)rows * d, st);
  }

  if (prefill) launch_seq_lens_set(cu_dev, batch, kv->seq_lens, st);
  else launch_seq_lens_inc(batch, c.max_seq, kv->seq_lens, st);
  if (timed) LS_HIP(hipEventRecord(s->pass_end, st));
  LS_HIP(hipGetLastError());
  return LS_OK;
}

// ---- host-side validation: everything a forward call can reject before it enqueues ------
ls_status check_state(const char* who, const ls_stage* s, int batch) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "%s: NULL stage", who);
  if (batch < 1 || batch > (int)s->cfg.max_batch)
    return fail(LS_ERR_INVALID_ARG, "%s: batch %d outside [1,%u]", who, batch, s->cfg.max_batch);
  for (const auto& b : s->blocks)
    if (b.state == NOT_LOADED) return fail(LS_ERR_NOT_LOADED, "%s: block %d has not been enqueued for load", who, b.layer);
  return LS_OK;
}

ls_status check_prefill(const char* who, const ls_stage* s, const int32_t* cu_host, int batch, int total_tokens,
                        int* max_len_out) {
  ls_status rc = check_state(who, s, batch);
  if (rc != LS_OK) return rc;
  if (!cu_host) return fail(LS_ERR_INVALID_ARG, "%s: NULL cu_seqlens", who);
  if (total_tokens < batch || total_tokens > (int)s->cfg.max_tokens)
    return fail(LS_ERR_INVALID_ARG, "%s: total_tokens %d outside [%d,%u]", who, total_tokens, batch, s->cfg.max_tokens);
  if (cu_host[0] != 0 || cu_host[batch] != total_tokens)
    return fail(LS_ERR_INVALID_ARG, "%s: cu_seqlens must start at 0 and end at total_tokens", who);
  int max_len = 0;
  for (int b = 0; b < batch; ++b) {
    int len = cu_host[b + 1] - cu_host[b];
    if (len > max_len) max_len = len;
    if (len < 1) return fail(LS_ERR_INVALID_ARG, "%s: sequence %d has length %d", who, b, len);
    if (len > (int)s->cfg.max_seq)
      return fail(LS_ERR_KV_OVERFLOW, "%s: sequence %d has %d tokens, max_seq is %u", who, b, len, s->cfg.max_seq);
  }
  if (max_len_out) *max_len_out = max_len;
  return LS_OK;
}

ls_status check_decode(const char* who, const ls_stage* s, int batch, int max_ctx) {
  ls_status rc = check_state(who, s, batch);
  if (rc != LS_OK) return rc;
  if (max_ctx < 0) return fail(LS_ERR_INVALID_ARG, "%s: max_ctx %d is negative", who, max_ctx);
  if (max_ctx + 1 > (int)s->cfg.max_seq)
    return fail(LS_ERR_KV_OVERFLOW, "%s: context %d + 1 exceeds max_seq %u", who, max_ctx, s->cfg.max_seq);
  return LS_OK;
}

ls_status check_pointers(const char* who, const ls_stage* s, const void* in, const ls_kv* kv, const void* out,
                         const float* logits_out) {
  if (!s || !in || !kv || !out) return fail(LS_ERR_INVALID_ARG, "%s: NULL argument", who);
  if (!kv->k || !kv->v || !kv->seq_lens) return fail(LS_ERR_INVALID_ARG, "%s: NULL pointer inside ls_kv", who);
  if (logits_out && !s->last) return fail(LS_ERR_INVALID_ARG, "%s: logits_out given but the stage has no LM head", who);
  return LS_OK;
}

ls::GemmScratch workspace_scratch(const ls_stage* s) {
  ls::GemmScratch g;
  g.splitk = s->w.splitk_bytes ? (float*)(s->ws + s->w.splitk) : nullptr;
  g.bytes = s->w.splitk_bytes;
  return g;
}

// Largest split-K scratch any GEMM of one decode step over `rows` rows asks for.
size_t decode_scratch_need(const ls_stage* s, int rows) {
  const ls_cfg& c = s->cfg;
  if (c.dtype != LS_DTYPE_BF16 || rows <= 16) return 0;
  const int d = c.hidden, F = c.ffn, qd = c.n_q_heads * c.head_dim;
  const int qkv_cols = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  size_t need = 0;
  auto one = [&](int N, int K, bool glu) {
    if (!ls::gemm_wide_supported(rows, N, K)) return;
    const size_t b = ls::gemm_wide_workspace_bytes(rows, N, K, glu);
    if (b > need) need = b;
  };
  one(qkv_cols, d, false);
  one(d, qd, false);
  one(F, d, true);
  one(d, F, false);
  if (s->last) one((int)c.vocab, d, false);
  return need;
}

}  // namespace

extern "C" {

ls_status ls_stage_check_prefill(const ls_stage* s, const int32_t* cu_host, int batch, int total_tokens) {
  return check_prefill("ls_stage_check_prefill", s, cu_host, batch, total_tokens, nullptr);
}

ls_status ls_stage_check_decode(const ls_stage* s, int batch, int max_ctx) {
  return check_decode("ls_stage_check_decode", s, batch, max_ctx);
}

ls_status ls_stage_prefill(ls_stage* s, const void* in, const int32_t* cu_dev, const int32_t* cu_host, int batch,
                           int total_tokens, const ls_kv* kv, void* out, float* logits_out, void* hip_stream) {
  ls_status rc = check_pointers("ls_stage_prefill", s, in, kv, out, logits_out);
  if (rc != LS_OK) return rc;
  if (!cu_dev) return fail(LS_ERR_INVALID_ARG, "ls_stage_prefill: NULL cu_seqlens");
  int max_len = 0;
  rc = check_prefill("ls_stage_prefill", s, cu_host, batch, total_tokens, &max_len);
  if (rc != LS_OK) return rc;
  return forward(s, true, in, cu_dev, batch, total_tokens, max_len, kv, out, logits_out, (hipStream_t)hip_stream,
                 workspace_scratch(s));
}

ls_status ls_stage_decode(ls_stage* s, const void* in, int batch, int max_ctx, const ls_kv* kv, void* out,
                          float* logits_out, void* hip_stream) {
  ls_status rc = check_pointers("ls_stage_decode", s, in, kv, out, logits_out);
  if (rc != LS_OK) return rc;
  rc = check_decode("ls_stage_decode", s, batch, max_ctx);
  if (rc != LS_OK) return rc;
  // max_len of a decode step: the keys a row may attend to (cached ones plus its own)
  return forward(s, false, in, nullptr, batch, batch, max_ctx + 1, kv, out, logits_out, (hipStream_t)hip_stream,
                 workspace_scratch(s));
}

ls_status ls_stage_decode_static(ls_stage* s, const void* in, int batch, int max_ctx, const ls_kv* kv, void* out,
                                 float* logits_out, void* hip_stream) {
  ls_status rc = check_pointers("ls_stage_decode_static", s, in, kv, out, logits_out);
  if (rc != LS_OK) return rc;
  rc = check_decode("ls_stage_decode_static", s, batch, max_ctx);
  if (rc != LS_OK) return rc;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != s->device)
    return fail(LS_ERR_INVALID_ARG, "ls_stage_decode_static: the stage's device (%d) is not the current one", s->device);
  const size_t need = decode_scratch_need(s, batch);
  if (need > (size_t)LS_STATIC_SCRATCH_BYTES)
    return fail(LS_ERR_OOM, "ls_stage_decode_static: this step needs %zu bytes of scratch, the static array holds %zu",
                need, (size_t)LS_STATIC_SCRATCH_BYTES);
  // the K-split partials of this step go to the device's static array: every workgroup writes
  // its whole partial tile before the finishing kernel reads it, so nothing has to start at zero
  ls::GemmScratch g;
  g.splitk = (float*)s->static_scratch;
  g.bytes = LS_STATIC_SCRATCH_BYTES;
  return forward(s, false, in, nullptr, batch, batch, max_ctx + 1, kv, out, logits_out, (hipStream_t)hip_stream, g);
}

ls_status ls_stage_layer_times(ls_stage* s, float* copy_ms, float* compute_ms, float* copy_end_ms,
                               float* compute_end_ms, int n) {
  if (!s || n < 0 || n > s->hi - s->lo) return fail(LS_ERR_INVALID_ARG, "ls_stage_layer_times: bad arguments");
  const bool want_copy = copy_ms || copy_end_ms, want_comp = compute_ms || compute_end_ms;
  if (want_comp && !s->compute_timed)
    return fail(LS_ERR_INVALID_ARG, "ls_stage_layer_times: no prefill was recorded with profiling on");
  hipEvent_t origin = s->origin_block >= 0 ? s->blocks[s->origin_block].copy_start
                                           : (s->compute_timed ? s->comp_start[0] : nullptr);
  for (int i = 0; i < n; ++i) {
    const Block& b = s->blocks[s->layer0 + i];
    if (want_copy) {
      if (!b.timed) return fail(LS_ERR_INVALID_ARG, "ls_stage_layer_times: block %d was not copied with profiling on", b.layer);
      if (copy_ms) LS_HIP(hipEventElapsedTime(&copy_ms[i], b.copy_start, b.loaded));
      if (copy_end_ms) LS_HIP(hipEventElapsedTime(&copy_end_ms[i], origin, b.loaded));
    }
    if (compute_ms) LS_HIP(hipEventElapsedTime(&compute_ms[i], s->comp_start[i], s->comp_end[i]));
    if (compute_end_ms) LS_HIP(hipEventElapsedTime(&compute_end_ms[i], origin, s->comp_end[i]));
  }
  return LS_OK;
}

ls_status ls_stage_block_times(ls_stage* s, int layer, float* copy_ms, float* copy_end_ms) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_block_times: NULL stage");
  const Block* b = s->find(layer);
  if (!b) return fail(LS_ERR_BLOCK_RANGE, "ls_stage_block_times: block %d is not held by stage [%d,%d)", layer, s->lo, s->hi);
  if (!b->timed || s->origin_block < 0)
    return fail(LS_ERR_INVALID_ARG, "ls_stage_block_times: block %d was not copied with profiling on", layer);
  if (copy_ms) LS_HIP(hipEventElapsedTime(copy_ms, b->copy_start, b->loaded));
  if (copy_end_ms) LS_HIP(hipEventElapsedTime(copy_end_ms, s->blocks[s->origin_block].copy_start, b->loaded));
  return LS_OK;
}

ls_status ls_stage_pass_times(ls_stage* s, float* before_layers_ms, float* after_layers_ms, float* total_ms) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_pass_times: NULL stage");
  if (!s->compute_timed) return fail(LS_ERR_INVALID_ARG, "ls_stage_pass_times: no prefill was recorded with profiling on");
  if (before_layers_ms) LS_HIP(hipEventElapsedTime(before_layers_ms, s->pass_start, s->comp_start[0]));
  if (after_layers_ms) LS_HIP(hipEventElapsedTime(after_layers_ms, s->comp_end.back(), s->pass_end));
  if (total_ms) LS_HIP(hipEventElapsedTime(total_ms, s->pass_start, s->pass_end));
  return LS_OK;
}

ls_status ls_stage_probe(ls_stage* s, int op, int layer, int phase) {
  if (!s) return fail(LS_ERR_INVALID_ARG, "ls_stage_probe: NULL stage");
  if (op < LS_OP_NONE || op > LS_OP_GEMM_DOWN || (phase != 0 && phase != 1))
    return fail(LS_ERR_INVALID_ARG, "ls_stage_probe: bad operator %d or phase %d", op, phase);
  if (op != LS_OP_NONE && (layer < s->lo || layer >= s->hi))
    return fail(LS_ERR_BLOCK_RANGE, "ls_stage_probe: layer %d outside [%d,%d)", layer, s->lo, s->hi);
  if (op != LS_OP_NONE && s->probe_a.empty()) {
    for (int i = 0; i < PROBE_CAP; ++i) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        if (a) (void)hipEventDestroy(a);
        return fail(LS_ERR_HIP, "ls_stage_probe: hipEventCreate failed");
      }
      s->probe_a.push_back(a);
      s->probe_b.push_back(b);
    }
    for (int i = 0; i < PROBE_CAP; ++i) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        if (a) (void)hipEventDestroy(a);
        return fail(LS_ERR_HIP, "ls_stage_probe: hipEventCreate failed");
      }
      s->probe_ka.push_back(a);
      s->probe_kb.push_back(b);
    }
    s->probe_exact.assign(PROBE_CAP, 0);
  }
  s->probe_op = op;
  s->probe_layer = layer;
  s->probe_phase = phase;
  if (op != LS_OP_NONE) s->probe_count = 0;  // switching off keeps what was recorded readable
  return LS_OK;
}

ls_status ls_stage_workspace_region(const ls_stage* s, int which, size_t* offset, size_t* bytes) {
  if (!s || !offset || !bytes) return fail(LS_ERR_INVALID_ARG, "ls_stage_workspace_region: NULL argument");
  const ls_cfg& c = s->cfg;
  const size_t T = c.max_tokens, e = isz(&c);
  switch (which) {
    case LS_WS_QKV: *offset = s->w.qkv; *bytes = T * (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * e; break;
    case LS_WS_ATTN: *offset = s->w.attn; *bytes = T * (size_t)c.n_q_heads * c.head_dim * e; break;
    case LS_WS_FFN: *offset = s->w.h; *bytes = T * (size_t)c.ffn * e; break;
    default: return fail(LS_ERR_INVALID_ARG, "ls_stage_workspace_region: unknown region %d", which);
  }
  return LS_OK;
}

int ls_stage_probe_is_kernel_exact(const ls_stage* s) {
  if (!s || s->probe_exact.empty() || s->probe_count == 0) return 0;
  const size_t have = s->probe_count < (size_t)PROBE_CAP ? s->probe_count : (size_t)PROBE_CAP;
  for (size_t i = 0; i < have; ++i)
    if (!s->probe_exact[i]) return 0;
  return 1;
}

ls_status ls_stage_probe_times(ls_stage* s, float* ms, int cap, int* n) {
  if (!s || !ms || !n || cap < 0) return fail(LS_ERR_INVALID_ARG, "ls_stage_probe_times: bad arguments");
  size_t have = s->probe_count < (size_t)PROBE_CAP ? s->probe_count : (size_t)PROBE_CAP;
  if (have > (size_t)cap) have = (size_t)cap;
  for (size_t i = 0; i < have; ++i) {
    if (s->probe_exact[i]) LS_HIP(hipEventElapsedTime(&ms[i], s->probe_ka[i], s->probe_kb[i]));
    else LS_HIP(hipEventElapsedTime(&ms[i], s->probe_a[i], s->probe_b[i]));
  }
  *n = (int)have;
  return LS_OK;
}

}  // extern "C"
