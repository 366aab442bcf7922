// Host side of the C ABI declared in include/fleet.h: device probing, scratch
// allocation, graph upload and the per-step launch of the persistent kernel.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/fleet.h"
#include "graph.hpp"
#include "kernels.hip.inc"
#include "aux_kernels.hip.inc"

// The flavours of the persistent kernel are instantiated in translation units of their own
// (kernel_variant.hip, one per flavour, compiled in parallel); here only their addresses are used.
#define FLEET_EXTERN_VARIANT(V)                                                        \
  extern template __global__ void fleet_persistent_kernel<V, false>(dev::Params);     \
  extern template __global__ void fleet_persistent_kernel<V, true>(dev::Params);
FLEET_EXTERN_VARIANT(0) FLEET_EXTERN_VARIANT(1) FLEET_EXTERN_VARIANT(2) FLEET_EXTERN_VARIANT(3)
FLEET_EXTERN_VARIANT(4) FLEET_EXTERN_VARIANT(5) FLEET_EXTERN_VARIANT(6)
#undef FLEET_EXTERN_VARIANT

// Workspace of fleet_decode_step_static, the entry point that allocates nothing: the
// activations, partial sums, counters and status block of one step live in this array
// instead of the fleet's own allocation.  Host code never uses the array's name as an
// address: the device address is looked up once per device (static_workspace()).
static __device__ __align__(256) unsigned char fleet_static_scratch[FLEET_STATIC_SCRATCH_BYTES];

namespace {

using namespace fleetg;

constexpr size_t LDS_BYTES = 128 * 1024;  // > half of a CU's 160 KB: one worker per CU
constexpr int TRACE_CAP = 2048;           // records per worker
constexpr int MAX_DEVICES = 64;

struct DevInfo {
  int n_cu = 0, n_xcd = 0;
  int per_xcd[dev::MAX_XCD] = {0};
};

// Device memory one launch works in besides the caller's buffers and the graph's
// descriptors: activations, partial sums, the counter block and the status block, carved
// from one base (the fleet's own allocation, or the static workspace).
struct Work {
  float* x = nullptr; void* n = nullptr; float* qkv = nullptr; void* att = nullptr; void* h = nullptr;
  float* part = nullptr; float* gpart = nullptr; float* gu32 = nullptr;
  float* ss = nullptr;       // sums of squares of the residual rows, per 16 features
  uint32_t* ctr = nullptr; int32_t* status = nullptr;
  size_t gpart_region = 0;   // bytes between the per-XCD regions of gpart
};

struct DevGraph {
  Graph g;
  int32_t *ops = nullptr, *tasks = nullptr, *events = nullptr, *qoff = nullptr, *qents = nullptr;
  int32_t* fat = nullptr;   // [n_tasks][FAT_WORDS]: task words, op words, weight pointers, id
  int ctr_words = 0, gcnt_base = 0;
  ~DevGraph() {
    for (void* p : {(void*)ops, (void*)tasks, (void*)events, (void*)qoff, (void*)qents, (void*)fat})
      if (p) (void)hipFree(p);
  }
};

thread_local int g_last_hip = 0;
#define HIP_TRY(expr)                              \
  do {                                             \
    hipError_t e_ = (expr);                        \
    if (e_ != hipSuccess) {                        \
      g_last_hip = (int)e_;                        \
      return e_ == hipErrorOutOfMemory ? FLEET_ENOMEM : FLEET_EHIP; \
    }                                              \
  } while (0)

template <class T>
int upload(T** dst, const void* src, size_t bytes) {
  *dst = nullptr;
  if (bytes == 0) bytes = 16;
  HIP_TRY(hipMalloc((void**)dst, bytes));
  if (src) HIP_TRY(hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice));
  return FLEET_OK;
}

// *dst = new device buffer holding the [rows][K] bf16 matrix `src` as MFMA operand blocks
int pack_matrix(void** dst, const void* src, int rows, int K, bool by_unit) {
  const int nrb = (rows + 15) / 16;
  const size_t bytes = (size_t)nrb * 16 * K * 2;
  HIP_TRY(hipMalloc(dst, bytes));
  hipLaunchKernelGGL(fleet_pack_kernel, dim3(2048), dim3(256), 0, 0, (const u32x4*)src, (u32x4*)*dst, rows, nrb, K, by_unit ? 1 : 0);
  HIP_TRY(hipGetLastError());
  return FLEET_OK;
}

// the persistent kernel compiled for one GEMM flavour (see dev::N_VARIANTS)
const void* kernel_variant(int v, bool paged = false) {
  if (paged) {
    switch (v) {
      case 0: return (const void*)fleet_persistent_kernel<0, true>;
      case 1: return (const void*)fleet_persistent_kernel<1, true>;
      case 2: return (const void*)fleet_persistent_kernel<2, true>;
      case 3: return (const void*)fleet_persistent_kernel<3, true>;
      case 4: return (const void*)fleet_persistent_kernel<4, true>;
      case 5: return (const void*)fleet_persistent_kernel<5, true>;
      default: return (const void*)fleet_persistent_kernel<6, true>;
    }
  }
  switch (v) {
    case 0: return (const void*)fleet_persistent_kernel<0>;
    case 1: return (const void*)fleet_persistent_kernel<1>;
    case 2: return (const void*)fleet_persistent_kernel<2>;
    case 3: return (const void*)fleet_persistent_kernel<3>;
    case 4: return (const void*)fleet_persistent_kernel<4>;
    case 5: return (const void*)fleet_persistent_kernel<5>;
    default: return (const void*)fleet_persistent_kernel<6>;
  }
}
// variant for a graph: FMA path by batch (1, 2, 4, 8), MFMA path by tile height
int variant_for(int path, int batch, int tile_m) {
  if (path == P_FMA) return batch <= 1 ? 0 : batch <= 2 ? 1 : batch <= 4 ? 2 : 3;
  return tile_m <= 16 ? 4 : tile_m <= 32 ? 5 : 6;
}
int launch_persistent(DevGraph* dg, dev::Params& P, int n_cu, hipStream_t st) {
  const Graph& g = dg->g;
  const int v = variant_for(g.header[H_PATH], g.header[H_BATCH], g.header[H_TILE_M]);
  void* args[] = {(void*)&P};
  HIP_TRY(hipLaunchKernel(kernel_variant(v, P.page_size > 0), dim3(n_cu), dim3(dev::WG), args, LDS_BYTES, st));
  return FLEET_OK;
}

// Per-device, once: raise the kernels' dynamic LDS limit and check that one worker fits a CU.
std::mutex g_dev_mutex;
bool g_prepared[MAX_DEVICES] = {false};
void* g_static_ws[MAX_DEVICES] = {nullptr};

int prepare_kernel() {
  int dev_id = 0, lds = 0;
  HIP_TRY(hipGetDevice(&dev_id));
  if (dev_id < 0 || dev_id >= MAX_DEVICES) return FLEET_EDEVICE;
  std::lock_guard<std::mutex> lock(g_dev_mutex);
  if (g_prepared[dev_id]) return FLEET_OK;
  HIP_TRY(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev_id));
  if ((size_t)lds < LDS_BYTES + 4096) return FLEET_EDEVICE;
  for (int v = 0; v < dev::N_VARIANTS; ++v) {
    HIP_TRY(hipFuncSetAttribute(kernel_variant(v), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES));
    HIP_TRY(hipFuncSetAttribute(kernel_variant(v, true), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES));
  }
  HIP_TRY(hipFuncSetAttribute((const void*)fleet_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES));
  int per_cu = 0;
  HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fleet_persistent_kernel<6>, dev::WG, LDS_BYTES));
  if (per_cu < 1) return FLEET_EDEVICE;
  g_prepared[dev_id] = true;
  return FLEET_OK;
}

// Device address of the static workspace on the current device (every device holds its own
// copy of the array at its own address); looked up once per device.
int static_workspace(void** out) {
  int dev_id = 0;
  HIP_TRY(hipGetDevice(&dev_id));
  if (dev_id < 0 || dev_id >= MAX_DEVICES) return FLEET_EDEVICE;
  std::lock_guard<std::mutex> lock(g_dev_mutex);
  if (!g_static_ws[dev_id]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(fleet_static_scratch)));
    if (!p) return FLEET_EHIP;
    g_static_ws[dev_id] = p;
  }
  *out = g_static_ws[dev_id];
  return FLEET_OK;
}

int probe_device(DevInfo* info, int32_t* xcd_of_block_out, int n_blocks_req) {
  int rc = prepare_kernel();
  if (rc) return rc;
  int dev_id = 0, n_cu = 0;
  HIP_TRY(hipGetDevice(&dev_id));
  HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev_id));
  int n_blocks = n_blocks_req > 0 ? n_blocks_req : n_cu;
  int32_t* d = nullptr;
  HIP_TRY(hipMalloc((void**)&d, sizeof(int32_t) * n_blocks));
  hipLaunchKernelGGL(fleet_probe_kernel, dim3(n_blocks), dim3(dev::WG), LDS_BYTES, 0, d);
  std::vector<int32_t> h(n_blocks);
  hipError_t e = hipMemcpy(h.data(), d, sizeof(int32_t) * n_blocks, hipMemcpyDeviceToHost);
  (void)hipFree(d);
  HIP_TRY(e);
  if (info) {
    info->n_cu = n_cu;
    info->n_xcd = 0;
    for (int x = 0; x < dev::MAX_XCD; ++x) info->per_xcd[x] = 0;
    for (int i = 0; i < n_blocks; ++i) {
      if (h[i] < 0 || h[i] >= dev::MAX_XCD) return FLEET_EDEVICE;
      info->per_xcd[h[i]]++;
      info->n_xcd = std::max(info->n_xcd, h[i] + 1);
    }
  }
  if (xcd_of_block_out) memcpy(xcd_of_block_out, h.data(), sizeof(int32_t) * n_blocks);
  return FLEET_OK;
}

long long timeout_ticks_from_env() {
  double ms = 2000.0;
  if (const char* s = getenv("FLEET_TIMEOUT_MS")) { double v = atof(s); if (v > 0) ms = v; }
  return (long long)(ms * 1e5);   // 100 MHz
}

constexpr size_t WORK_ALIGN = 256;
size_t align_up(size_t v) { return (v + WORK_ALIGN - 1) / WORK_ALIGN * WORK_ALIGN; }

}  // namespace

struct fleet {
  fleet_shape_t shape;
  int fma_max = 2;   // largest batch on the FMA GEMV path, latched at create
  std::vector<const void*> ln1, wqkv, q_norm, k_norm, wo, ln2, wgu, wdown;
  const void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
  // library-owned copies of the GEMM weights in the operand-block layout of the MFMA
  // kernels (made by fleet_create when max_batch reaches those kernels)
  std::vector<void*> pk_qkv, pk_o, pk_gu, pk_down;
  void* pk_lm = nullptr;
  DevInfo info;
  // one graph per batch bucket, built and uploaded by fleet_create: a step of `batch`
  // sequences runs the graph of the smallest bucket that holds it
  std::vector<int> buckets;
  std::vector<std::unique_ptr<DevGraph>> graphs;        // by bucket
  std::vector<std::unique_ptr<DevGraph>> graphs_loop;   // with the next-token stage (multi-step launches)
  char* work = nullptr;      // the fleet's own working memory (layout: work_layout())
  size_t work_bytes = 0;
  float2* rope = nullptr;
  int32_t* trace = nullptr;
  long long timeout_ticks = 0;
  int32_t* last_status = nullptr;   // status block of the last launch (device)
  float* last_x = nullptr;          // residual stream of the last launch (device)

  ~fleet() {
    for (void* p : {(void*)work, (void*)rope, (void*)trace})
      if (p) (void)hipFree(p);
    for (auto* v : {&pk_qkv, &pk_o, &pk_gu, &pk_down})
      for (void* p : *v) if (p) (void)hipFree(p);
    if (pk_lm) (void)hipFree(pk_lm);
  }
};

namespace {

// Working memory of one launch of graph dg, carved from `base` (may be null: sizes only).
// Returns the bytes needed.
size_t work_layout(const fleet* f, const DevGraph* dg, char* base, Work* w) {
  const Graph& g = dg->g;
  const fleet_shape_t& s = f->shape;
  const size_t B = g.header[H_BATCH], B16 = (B + 15) / 16 * 16, H = s.hidden, F = s.ffn;
  const size_t NQKV = (size_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim, QD = (size_t)s.n_q_heads * s.head_dim;
  const size_t grp = s.n_q_heads / s.n_kv_heads, S = std::max(1, g.header[H_N_SPLITS]);
  auto pad256 = [](size_t k) { return (k + 255) / 256 * 256; };
  // partial sums of the graph's split-K operators: [k-slice][unit][m-tile][blocks x 256] fp32
  size_t gp = 0;
  for (int i = 0; i < g.n_ops(); ++i) {
    const int32_t* o = &g.ops[(size_t)i * OP_WORDS];
    if (o[O_BODY] != B_GEMM || o[O_PATH] != P_MFMA) continue;
    const size_t ks = std::max(1, (o[O_AUX2] >> 16) & 15), nb = o[O_EPI] == E_SWIGLU_BF16 ? 2 : 1;
    if (ks > 1) gp = std::max(gp, ks * nb * (size_t)o[O_N_UNITS] * o[O_M_TILES] * mfma_blocks(o[O_TILE_M]) * 256 * 4);
  }
  gp = align_up(gp);
  const size_t regions = s.sched_mode == FLEET_SCHED_UNAWARE ? 1 : dev::MAX_XCD;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += align_up(bytes); return p; };
  char* x = take(B * H * 4);
  char* n = take(B16 * pad256(H) * 2);       // bf16 activations: operand blocks of 16 rows on the MFMA path
  char* qkv = take(B * NQKV * 4);
  char* att = take(B16 * pad256(QD) * 2);
  char* h = take(B16 * pad256(F) * 2);
  char* part = take(B * s.n_kv_heads * S * grp * dev::PART_STRIDE * 4);
  char* gpart = take(gp * regions);
  char* gu32 = take((s.flags & FLEET_FLAG_UNFUSED_SILU) ? B * 2 * F * 4 : 0);
  char* ss = take(B * (H / 16) * 4);
  char* ctr = take((size_t)dg->ctr_words * 4);
  char* status = take(dev::ST_WORDS * 4);
  if (w) {
    w->x = (float*)x; w->n = n; w->qkv = (float*)qkv; w->att = att; w->h = h; w->part = (float*)part;
    w->gpart = (float*)gpart; w->gu32 = (float*)gu32; w->ss = (float*)ss; w->ctr = (uint32_t*)ctr; w->status = (int32_t*)status;
    w->gpart_region = gp;
  }
  return off;
}

int resolve_weight(const fleet* f, int wkind, int layer, const void* const* gemm_copies, bool packed,
                   const void** first, const void** second) {
  *first = *second = nullptr;
  if (packed && f) {
    const std::vector<void*>* v = nullptr;
    switch (wkind) {
      case W_QKV: v = &f->pk_qkv; break;
      case W_O: v = &f->pk_o; break;
      case W_GU: v = &f->pk_gu; break;
      case W_DOWN: v = &f->pk_down; break;
      case W_LM: if (!f->pk_lm) return FLEET_EINVAL; *first = f->pk_lm; return FLEET_OK;
      default: break;
    }
    if (v) {   // an MFMA graph needs the packed copies fleet_create makes
      if ((size_t)layer >= v->size() || !(*v)[layer]) return FLEET_EINVAL;
      *first = (*v)[layer];
      return FLEET_OK;
    }
  }
  switch (wkind) {
    case W_QKV: *first = f->wqkv[layer]; break;
    case W_O: *first = f->wo[layer]; break;
    case W_GU: *first = f->wgu[layer]; break;
    case W_DOWN: *first = f->wdown[layer]; break;
    case W_LM: *first = f->lm_head; break;
    case W_LN1: *first = f->ln1[layer]; break;
    case W_LN2: *first = f->ln2[layer]; break;
    case W_FINAL: *first = f->final_norm; break;
    case W_EMBED: *second = f->embed; break;
    case W_GEMM_COPY: *first = gemm_copies ? gemm_copies[layer] : nullptr; break;
    default: break;
  }
  return FLEET_OK;
}

int upload_graph(DevGraph* dg, const fleet* f, const void* const* gemm_copies, int n_xcd) {
  const Graph& g = dg->g;
  int rc;
  if ((rc = upload(&dg->ops, g.ops.data(), g.ops.size() * 4))) return rc;
  if ((rc = upload(&dg->tasks, g.tasks.data(), g.tasks.size() * 4))) return rc;
  if ((rc = upload(&dg->events, g.events.data(), g.events.size() * 4))) return rc;
  if ((rc = upload(&dg->qoff, g.qoff.data(), g.qoff.size() * 4))) return rc;
  if ((rc = upload(&dg->qents, g.qents.data(), g.qents.size() * 4))) return rc;
  std::vector<const void*> w(g.n_ops()), w2(g.n_ops());
  for (int i = 0; i < g.n_ops(); ++i) {
    const int32_t* o = &g.ops[(size_t)i * OP_WORDS];
    if (o[O_BODY] == B_ATTN && f) { w[i] = f->q_norm[o[O_LAYER]]; w2[i] = f->k_norm[o[O_LAYER]]; continue; }
    if (!f && !gemm_copies) continue;
    const void *first = nullptr, *second = nullptr;
    if ((rc = resolve_weight(f, o[O_WKIND], o[O_LAYER], gemm_copies, o[O_PATH] == P_MFMA, &first, &second))) return rc;
    if (o[O_BODY] == B_GEMM && (o[O_AUX2] & 0xff) != W_NONE && f) {   // gain of the fused RMSNorm, or the matrix to warm
      const void* unused = nullptr;
      if ((rc = resolve_weight(f, o[O_AUX2] & 0xff, o[O_LAYER], nullptr, false, &second, &unused))) return rc;
    }
    w[i] = first; w2[i] = second;
  }
  // one self-contained descriptor per task, so that a worker fetches it with one read
  std::vector<int32_t> fat((size_t)g.n_tasks() * dev::FAT_WORDS, 0);
  for (int t = 0; t < g.n_tasks(); ++t) {
    int32_t* d = &fat[(size_t)t * dev::FAT_WORDS];
    const int32_t* tw = &g.tasks[(size_t)t * TASK_WORDS];
    memcpy(d, tw, TASK_WORDS * 4);
    memcpy(d + TASK_WORDS, &g.ops[(size_t)tw[T_OP] * OP_WORDS], OP_WORDS * 4);
    memcpy(d + dev::FAT_W, &w[tw[T_OP]], sizeof(void*));
    memcpy(d + dev::FAT_W2, &w2[tw[T_OP]], sizeof(void*));
    d[dev::FAT_ID] = t;
  }
  // CU-tasks dealt inside one XCD: how many of them signal the task's event from that XCD
  for (int x = 0; x < n_xcd; ++x)
    for (int qi = g.qoff[x]; qi < g.qoff[x + 1]; ++qi) {
      const int32_t* e = &g.qents[(size_t)qi * QENT_WORDS];
      if (e[Q_DIST] != D_XCD_RR && e[Q_DIST] != D_XCD_RR_TOP) continue;
      for (int t = e[Q_FIRST]; t < e[Q_FIRST] + e[Q_COUNT]; ++t) fat[(size_t)t * dev::FAT_WORDS + dev::FAT_GROUP] = e[Q_COUNT];
    }
  if ((rc = upload(&dg->fat, fat.data(), fat.size() * 4))) return rc;
  // counter block: G[e], L[x][e], one arrival counter per (sequence, kv head) for the split-KV
  // merge, the per-XCD copies of the device counters (rows on their own cache lines), and
  // (MFMA graphs) the arrival counters of split-K GEMM tiles
  if (g.n_events() > dev::ECACHE) return FLEET_EINVAL;   // the kernel keeps one table entry per event in LDS
  dg->gcnt_base = dev::C_EVENTS + g.n_events() * (1 + n_xcd) + dev::N_PAIR +
                  dev::COPY_GROUPS * n_xcd * ((g.n_events() + 31) & ~31);
  dg->ctr_words = dg->gcnt_base + (g.header[H_PATH] == P_MFMA ? dev::GEMM_CNT_WORDS : 0);
  return FLEET_OK;
}

// reset counters and status, then run queue slice [q_begin, q_end) of every XCD
int launch(dev::Params& P, DevGraph* dg, int n_cu, int preset_event, hipStream_t st) {
  const int words = dg->ctr_words;
  int preset_word = -1;
  uint32_t preset_val = 0;
  if (preset_event >= 0) {
    preset_word = dev::C_EVENTS + preset_event;
    preset_val = 0x40000000u;   // satisfied whatever the threshold
  }
  const int nE = dg->g.n_events(), nx = dg->g.header[H_N_XCD], cstride = (nE + 31) & ~31;
  const int cbase = dev::C_EVENTS + nE * (1 + nx) + dev::N_PAIR;
  hipLaunchKernelGGL(fleet_reset_kernel, dim3((words + 255) / 256), dim3(256), 0, st, P.ctr, words, preset_word,
                     preset_val, P.status, cbase, cstride, dev::COPY_GROUPS * nx, preset_event);
  return launch_persistent(dg, P, n_cu, st);
}

void fill_graph_params(dev::Params& P, const DevGraph* dg) {
  P.ops = dg->ops; P.tasks = dg->tasks; P.events = dg->events; P.qoff = dg->qoff; P.qents = dg->qents;
  P.fat = dg->fat; P.n_events = dg->g.n_events(); P.gcnt_base = dg->gcnt_base;
}

// the graph that serves a step of `batch` sequences: the smallest bucket that holds it
DevGraph* pick_graph(fleet* f, int batch, bool loop) {
  auto& set = loop ? f->graphs_loop : f->graphs;
  for (size_t i = 0; i < f->buckets.size() && i < set.size(); ++i)
    if (f->buckets[i] >= batch) return set[i].get();
  return nullptr;
}

struct KvPaging {   // paged KV cache: k_cache / v_cache are page pools
  const int32_t* table = nullptr;   // device [batch][stride] page indices
  int page_size = 0, n_pages = 0, stride = 0;
};

struct StepArgs {
  int batch = 0, layer_begin = 0, layer_end = 0;
  bool with_ingest = false, with_final = false;
  const void* hidden_in = nullptr; const int32_t* tokens = nullptr;
  void *k_cache = nullptr, *v_cache = nullptr; const int32_t* positions = nullptr;
  float *hidden_out = nullptr, *logits = nullptr;
  int n_tokens = 0; int32_t* tokens_out = nullptr;   // n_tokens > 0: that many steps in one launch
  const KvPaging* paging = nullptr;
  const float* x_in = nullptr;                       // layer ranges: residual stream to start from
  bool static_ws = false;                            // work in the static workspace
};

// No allocation, no host-device copy, no synchronisation: kernels (and, for layer ranges,
// device-to-device copies) on the stream only.
int run_layers(fleet* f, const StepArgs& a, hipStream_t st) {
  // the kernels move activations, cache rows and logits in 16-byte pieces
  for (const void* p : {a.hidden_in, (const void*)a.k_cache, (const void*)a.v_cache, (const void*)a.hidden_out, (const void*)a.logits})
    if ((uintptr_t)p % 16 != 0) return FLEET_EINVAL;
  for (const void* p : {(const void*)a.tokens, (const void*)a.positions, (const void*)a.tokens_out, a.paging ? (const void*)a.paging->table : nullptr})
    if ((uintptr_t)p % 4 != 0) return FLEET_EINVAL;
  DevGraph* dg = pick_graph(f, a.batch, a.n_tokens > 0);
  if (!dg) return FLEET_EINVAL;
  const Graph& g = dg->g;
  Work w;
  if (a.static_ws) {
    if (work_layout(f, dg, nullptr, nullptr) > (size_t)FLEET_STATIC_SCRATCH_BYTES) return FLEET_ETOOBIG;
    void* base = nullptr;
    int rc = static_workspace(&base);   // looked up by fleet_create on this device: a table read here
    if (rc) return rc;
    work_layout(f, dg, (char*)base, &w);
  } else {
    work_layout(f, dg, f->work, &w);
  }
  const int L = f->shape.n_layers, nm = n_marks(L), nx = f->info.n_xcd;
  dev::Params P;
  memset(&P, 0, sizeof(P));
  fill_graph_params(P, dg);
  P.ctr = w.ctr; P.status = w.status;
  P.buf[BUF_X] = w.x; P.buf[BUF_N] = w.n; P.buf[BUF_QKV] = w.qkv; P.buf[BUF_ATT] = w.att; P.buf[BUF_H] = w.h;
  P.buf[BUF_PART] = w.part; P.buf[BUF_GPART] = w.gpart; P.buf[BUF_GU32] = w.gu32; P.buf[BUF_SS] = w.ss;
  P.buf[BUF_HIDDEN_IN] = (void*)a.hidden_in; P.buf[BUF_TOKENS] = (void*)a.tokens;
  P.buf[BUF_KC] = a.k_cache; P.buf[BUF_VC] = a.v_cache; P.buf[BUF_POS] = (void*)a.positions;
  P.buf[BUF_HIDDEN_OUT] = a.hidden_out; P.buf[BUF_LOGITS] = a.logits; P.buf[BUF_TOKENS_OUT] = a.tokens_out;
  P.n_iter = a.n_tokens > 0 ? a.n_tokens : 1;
  P.gpart_xcd_bytes = f->shape.sched_mode == FLEET_SCHED_UNAWARE ? 0 : (int32_t)w.gpart_region;
  if (a.paging) {
    P.buf[BUF_PT] = (void*)a.paging->table;
    P.page_size = a.paging->page_size; P.n_pages = a.paging->n_pages; P.pt_stride = a.paging->stride;
  }
  P.trace_cap = TRACE_CAP;
  // (no trace of a multi-step launch: the record area holds one step)
  P.trace = (a.n_tokens == 0 && (f->shape.flags & (FLEET_FLAG_TRACE | FLEET_FLAG_TIMING))) ? f->trace : nullptr;
  P.rope = f->rope; P.timeout_ticks = f->timeout_ticks; P.n_xcd = nx; P.flags = f->shape.flags;
  P.nq = f->shape.n_q_heads; P.nkv = f->shape.n_kv_heads; P.hd = f->shape.head_dim; P.max_batch = f->shape.max_batch;
  P.max_seq = f->shape.max_seq; P.hidden = f->shape.hidden; P.ffn = f->shape.ffn; P.batch = a.batch; P.eps = f->shape.rms_eps; P.vocab = f->shape.vocab;
  // marks of a queue: ingest, layer 0 .. L-1, final stage, LM head, end.  The final stage
  // (hidden_out, final norm) runs whenever asked for; the LM head only with a logits buffer.
  const int mb = a.with_ingest ? 0 : 1 + a.layer_begin;
  const int me = !a.with_final ? 1 + a.layer_end : (a.logits ? L + 3 : L + 2);
  for (int x = 0; x < nx; ++x) {
    P.q_begin[x] = g.marks[(size_t)x * nm + mb];
    P.q_end[x] = g.marks[(size_t)x * nm + me];
  }
  if (a.x_in) {   // a residual stream from the caller: copy it in, with the sums of squares its first consumer needs
    HIP_TRY(hipMemcpyAsync(w.x, a.x_in, (size_t)a.batch * f->shape.hidden * 4, hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(fleet_row_ss_kernel, dim3(std::max(1, a.batch * (f->shape.hidden / 16) / 256)), dim3(256), 0, st,
                       (const float*)w.x, w.ss, a.batch, f->shape.hidden);
  }
  const int preset = a.with_ingest ? -1 : g.xready[a.layer_begin];
  f->last_status = w.status;
  f->last_x = w.x;
  return launch(P, dg, f->info.n_cu, preset, st);
}

// Launch every kernel flavour the fleet's graphs use once, on empty queues (the workers start
// up, find nothing to do and leave): the runtime's own set-up for a kernel -- scratch memory for
// spilled registers above all -- then happens in fleet_create, not in the first step that needs it.
int warm_kernels(fleet* f) {
  bool seen[dev::N_VARIANTS] = {false};
  for (auto& dgp : f->graphs) {
    DevGraph* dg = dgp.get();
    const int v = variant_for(dg->g.header[H_PATH], dg->g.header[H_BATCH], dg->g.header[H_TILE_M]);
    if (seen[v]) continue;
    seen[v] = true;
    Work w;
    work_layout(f, dg, f->work, &w);
    for (int paged = 0; paged < 2; ++paged) {
      dev::Params P;
      memset(&P, 0, sizeof(P));
      fill_graph_params(P, dg);
      P.n_events = 0;   // no event table to cache, no task to run
      P.ctr = w.ctr; P.status = w.status;
      P.n_iter = 1; P.n_xcd = f->info.n_xcd; P.flags = f->shape.flags & ~(FLEET_FLAG_TRACE | FLEET_FLAG_TIMING);
      P.timeout_ticks = f->timeout_ticks; P.batch = 1; P.hidden = f->shape.hidden;
      P.page_size = paged ? 64 : 0; P.n_pages = paged;
      int rc = launch(P, dg, f->info.n_cu, -1, nullptr);
      if (rc) return rc;
    }
  }
  HIP_TRY(hipDeviceSynchronize());
  return FLEET_OK;
}

int check_step_args(const fleet* f, int batch, const void* hidden_in, const int32_t* tokens, const void* kc, const void* vc,
                    const int32_t* positions, const float* hidden_out) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !kc || !vc || !positions || !hidden_out) return FLEET_EINVAL;
  if (!hidden_in && !(tokens && f->embed)) return FLEET_EINVAL;
  return FLEET_OK;
}

}  // namespace

extern "C" {

const char* fleet_strerror(int code) {
  switch (code) {
    case FLEET_OK: return "ok";
    case FLEET_EINVAL: return "invalid argument";
    case FLEET_ENOMEM: return "out of memory";
    case FLEET_EHIP: return "HIP call failed";
    case FLEET_ETIMEOUT: return "dependency wait timed out; step aborted";
    case FLEET_ESMALL: return "buffer too small";
    case FLEET_EDEVICE: return "device cannot hold the persistent grid";
    case FLEET_ETOOBIG: return "the step needs more working memory than the static workspace holds";
    default: return "unknown error";
  }
}

int fleet_device_probe(int32_t n_blocks, int32_t* xcd_of_block) {
  if (n_blocks < 1 || n_blocks > 4096 || !xcd_of_block) return FLEET_EINVAL;
  return probe_device(nullptr, xcd_of_block, n_blocks);
}

int fleet_create(const fleet_shape_t* shape, const fleet_weights_t* w, fleet_t** out) {
  if (!shape || !w || !out) return FLEET_EINVAL;
  *out = nullptr;
  int rc = check_shape(*shape);
  if (rc) return rc;
  const int L = shape->n_layers;
  if (!w->ln1 || !w->wqkv || !w->q_norm || !w->k_norm || !w->wo || !w->ln2 || !w->wgu || !w->wdown) return FLEET_EINVAL;
  for (int l = 0; l < L; ++l)
    if (!w->ln1[l] || !w->wqkv[l] || !w->q_norm[l] || !w->k_norm[l] || !w->wo[l] || !w->ln2[l] || !w->wgu[l] || !w->wdown[l])
      return FLEET_EINVAL;
  if (shape->vocab > 0 && (!w->final_norm || !w->lm_head)) return FLEET_EINVAL;
  std::unique_ptr<fleet> f(new (std::nothrow) fleet());   // its destructor frees what the steps below allocated
  if (!f) return FLEET_ENOMEM;
  f->shape = *shape;
  // the FMA / MFMA switch is latched here: the packed copies and every graph follow it
  f->fma_max = (shape->flags & FLEET_FLAG_PACKED_ONLY) ? 0 : fma_max_from_env();
  f->ln1.assign(w->ln1, w->ln1 + L); f->wqkv.assign(w->wqkv, w->wqkv + L); f->q_norm.assign(w->q_norm, w->q_norm + L);
  f->k_norm.assign(w->k_norm, w->k_norm + L); f->wo.assign(w->wo, w->wo + L); f->ln2.assign(w->ln2, w->ln2 + L);
  f->wgu.assign(w->wgu, w->wgu + L); f->wdown.assign(w->wdown, w->wdown + L);
  f->embed = w->embed; f->final_norm = w->final_norm; f->lm_head = w->lm_head;
  f->timeout_ticks = timeout_ticks_from_env();
  if ((rc = probe_device(&f->info, nullptr, 0))) return rc;
  for (int x = 0; x < f->info.n_xcd; ++x)
    if (f->info.per_xcd[x] == 0) return FLEET_EDEVICE;
  {   // the static workspace's address on this device, for fleet_decode_step_static
    void* ws = nullptr;
    if ((rc = static_workspace(&ws))) return rc;
  }

  const size_t H = shape->hidden, F = shape->ffn;
  const size_t NQKV = (size_t)(shape->n_q_heads + 2 * shape->n_kv_heads) * shape->head_dim;
  const size_t QD = (size_t)shape->n_q_heads * shape->head_dim;
  if (shape->max_batch > f->fma_max) {
    f->pk_qkv.assign(L, nullptr); f->pk_o.assign(L, nullptr); f->pk_gu.assign(L, nullptr); f->pk_down.assign(L, nullptr);
    for (int l = 0; l < L; ++l) {
      if ((rc = pack_matrix(&f->pk_qkv[l], f->wqkv[l], (int)NQKV, (int)H, true))) return rc;
      if ((rc = pack_matrix(&f->pk_o[l], f->wo[l], (int)H, (int)QD, true))) return rc;
      if ((rc = pack_matrix(&f->pk_gu[l], f->wgu[l], (int)(2 * F), (int)H, true))) return rc;
      if ((rc = pack_matrix(&f->pk_down[l], f->wdown[l], (int)H, (int)F, true))) return rc;
    }
    if (shape->vocab > 0 && (rc = pack_matrix(&f->pk_lm, f->lm_head, shape->vocab, (int)H, true))) return rc;
    HIP_TRY(hipDeviceSynchronize());
  }
  if (shape->flags & FLEET_FLAG_PACKED_ONLY) {   // the caller may free the matrices now: forget them
    for (auto* v : {&f->wqkv, &f->wo, &f->wgu, &f->wdown}) v->assign(L, nullptr);
    f->lm_head = nullptr;
  }
  // Batch buckets: powers of two, the last FMA batch, max_batch.  Every graph is built and
  // uploaded here, so that a step allocates and copies nothing.
  for (int b = 1; b < shape->max_batch; b *= 2) f->buckets.push_back(b);
  if (f->fma_max >= 1 && f->fma_max < shape->max_batch) f->buckets.push_back(f->fma_max);
  f->buckets.push_back(shape->max_batch);
  std::sort(f->buckets.begin(), f->buckets.end());
  f->buckets.erase(std::unique(f->buckets.begin(), f->buckets.end()), f->buckets.end());
  const bool can_loop = shape->vocab > 0 && f->embed && f->final_norm;
  for (int loop = 0; loop < (can_loop ? 2 : 1); ++loop)
    for (int b : f->buckets) {
      std::unique_ptr<DevGraph> dg(new (std::nothrow) DevGraph());
      if (!dg) return FLEET_ENOMEM;
      dg->g = build_decode_graph(f->shape, b, f->info.n_xcd, f->info.n_cu, loop != 0, f->fma_max);
      if ((rc = upload_graph(dg.get(), f.get(), nullptr, f->info.n_xcd))) return rc;
      f->work_bytes = std::max(f->work_bytes, work_layout(f.get(), dg.get(), nullptr, nullptr));
      (loop ? f->graphs_loop : f->graphs).push_back(std::move(dg));
    }
  if ((rc = upload(&f->work, nullptr, f->work_bytes))) return rc;
  if ((rc = warm_kernels(f.get()))) return rc;
  {   // a status block that reads "ok" before the first step
    Work w0;
    work_layout(f.get(), f->graphs[0].get(), f->work, &w0);
    HIP_TRY(hipMemset(w0.status, 0, dev::ST_WORDS * 4));
    f->last_status = w0.status; f->last_x = w0.x;
  }
  if (shape->flags & (FLEET_FLAG_TRACE | FLEET_FLAG_TIMING))
    if ((rc = upload(&f->trace, nullptr, ((size_t)f->info.n_cu * TRACE_CAP * 8 + f->info.n_cu) * 4))) return rc;
  // rotary table: angle = pos * theta^(-2i/d), evaluated in double
  {
    const int half = shape->head_dim / 2;
    std::vector<float2> tab((size_t)shape->max_seq * half);
    for (int i = 0; i < half; ++i) {
      const double inv = std::pow((double)shape->rope_theta, -2.0 * i / (double)shape->head_dim);
      for (int p = 0; p < shape->max_seq; ++p) {
        const double a = (double)p * inv;
        tab[(size_t)p * half + i] = make_float2((float)std::cos(a), (float)std::sin(a));
      }
    }
    if ((rc = upload(&f->rope, tab.data(), tab.size() * sizeof(float2)))) return rc;
  }
  *out = f.release();
  return FLEET_OK;
}

int fleet_destroy(fleet_t* f) {
  if (!f) return FLEET_OK;
  (void)hipDeviceSynchronize();
  delete f;
  return FLEET_OK;
}

int fleet_decode_step(fleet_t* f, int32_t batch, const void* hidden_in, const int32_t* tokens, void* k_cache,
                      void* v_cache, const int32_t* positions, float* hidden_out, float* logits, void* stream) {
  int rc = check_step_args(f, batch, hidden_in, tokens, k_cache, v_cache, positions, hidden_out);
  if (rc) return rc;
  StepArgs a;
  a.batch = batch; a.layer_end = f->shape.n_layers; a.with_ingest = a.with_final = true;
  a.hidden_in = hidden_in; a.tokens = tokens; a.k_cache = k_cache; a.v_cache = v_cache; a.positions = positions;
  a.hidden_out = hidden_out; a.logits = f->shape.vocab > 0 ? logits : nullptr;
  return run_layers(f, a, (hipStream_t)stream);
}

int fleet_decode_step_static(fleet_t* f, int32_t batch, const void* hidden_in, const int32_t* tokens, void* k_cache,
                             void* v_cache, const int32_t* positions, float* hidden_out, float* logits, void* stream) {
  int rc = check_step_args(f, batch, hidden_in, tokens, k_cache, v_cache, positions, hidden_out);
  if (rc) return rc;
  StepArgs a;
  a.batch = batch; a.layer_end = f->shape.n_layers; a.with_ingest = a.with_final = true;
  a.hidden_in = hidden_in; a.tokens = tokens; a.k_cache = k_cache; a.v_cache = v_cache; a.positions = positions;
  a.hidden_out = hidden_out; a.logits = f->shape.vocab > 0 ? logits : nullptr;
  a.static_ws = true;
  return run_layers(f, a, (hipStream_t)stream);
}

int fleet_decode_layers(fleet_t* f, int32_t batch, int32_t layer_begin, int32_t layer_end, const float* x_in,
                        void* k_cache, void* v_cache, const int32_t* positions, float* x_out, float* logits,
                        void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !k_cache || !v_cache || !positions || !x_in || !x_out) return FLEET_EINVAL;
  const int L = f->shape.n_layers;
  if (layer_begin < 0 || layer_end > L || layer_begin >= layer_end) return FLEET_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  StepArgs a;
  a.batch = batch; a.layer_begin = layer_begin; a.layer_end = layer_end;
  a.with_final = layer_end == L && logits && f->shape.vocab > 0;
  a.k_cache = k_cache; a.v_cache = v_cache; a.positions = positions; a.hidden_out = x_out; a.logits = logits; a.x_in = x_in;
  int rc = run_layers(f, a, st);
  if (rc) return rc;
  if (!a.with_final) HIP_TRY(hipMemcpyAsync(x_out, f->last_x, (size_t)batch * f->shape.hidden * 4, hipMemcpyDeviceToDevice, st));
  return FLEET_OK;
}

int fleet_decode_step_paged(fleet_t* f, int32_t batch, const void* hidden_in, const int32_t* tokens, void* k_pool,
                            void* v_pool, const int32_t* page_table, int32_t page_size, int32_t n_pages,
                            int32_t table_stride, const int32_t* positions, float* hidden_out, float* logits,
                            void* stream) {
  int rc = check_step_args(f, batch, hidden_in, tokens, k_pool, v_pool, positions, hidden_out);
  if (rc) return rc;
  if (!page_table) return FLEET_EINVAL;
  if (page_size < 64 || (page_size & (page_size - 1)) || n_pages < 1 || table_stride < 1) return FLEET_EINVAL;
  // the kernel addresses a page with 32-bit page arithmetic inside one layer's pool
  if ((int64_t)n_pages * f->shape.n_kv_heads * page_size > (int64_t)1 << 40) return FLEET_EINVAL;
  KvPaging pg;
  pg.table = page_table; pg.page_size = page_size; pg.n_pages = n_pages; pg.stride = table_stride;
  StepArgs a;
  a.batch = batch; a.layer_end = f->shape.n_layers; a.with_ingest = a.with_final = true;
  a.hidden_in = hidden_in; a.tokens = tokens; a.k_cache = k_pool; a.v_cache = v_pool; a.positions = positions;
  a.hidden_out = hidden_out; a.logits = f->shape.vocab > 0 ? logits : nullptr; a.paging = &pg;
  return run_layers(f, a, (hipStream_t)stream);
}

int fleet_decode_tokens(fleet_t* f, int32_t batch, int32_t* tokens, void* k_cache, void* v_cache, int32_t* positions,
                        int32_t n_tokens, int32_t* tokens_out, float* hidden_out, float* logits, void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !tokens || !k_cache || !v_cache || !positions || !tokens_out ||
      !hidden_out || !logits || n_tokens < 1 || n_tokens > 65536)
    return FLEET_EINVAL;
  if (f->shape.vocab <= 0 || !f->embed || !f->final_norm || f->graphs_loop.empty()) return FLEET_EINVAL;
  StepArgs a;
  a.batch = batch; a.layer_end = f->shape.n_layers; a.with_ingest = a.with_final = true;
  a.tokens = tokens; a.k_cache = k_cache; a.v_cache = v_cache; a.positions = positions;
  a.hidden_out = hidden_out; a.logits = logits; a.n_tokens = n_tokens; a.tokens_out = tokens_out;
  return run_layers(f, a, (hipStream_t)stream);
}

int fleet_last_status(fleet_t* f, fleet_status_t* out) {
  if (!f || !out) return FLEET_EINVAL;
  memset(out, 0, sizeof(*out));
  hipError_t e = hipDeviceSynchronize();
  out->hip_error = e != hipSuccess ? (int)e : g_last_hip;
  int32_t st[dev::ST_WORDS];
  HIP_TRY(hipMemcpy(st, f->last_status, sizeof(st), hipMemcpyDeviceToHost));
  out->code = e != hipSuccess ? FLEET_EHIP : st[dev::ST_CODE];
  out->task = st[dev::ST_TASK]; out->event = st[dev::ST_EVENT];
  out->observed = st[dev::ST_OBSERVED]; out->needed = st[dev::ST_NEEDED];
  out->n_xcd = f->info.n_xcd;
  for (int x = 0; x < 8; ++x) out->workers[x] = st[dev::ST_WORKERS + x];
  return FLEET_OK;
}

static int copy_words(const std::vector<int32_t>& words, void* buf, size_t* len) {
  const size_t need = words.size() * 4;
  if (!buf || *len < need) { *len = need; return buf ? FLEET_ESMALL : FLEET_OK; }
  memcpy(buf, words.data(), need);
  *len = need;
  return FLEET_OK;
}

int fleet_graph_build(const fleet_shape_t* shape, int32_t batch, int32_t n_xcd, int32_t n_workers, void* buf, size_t* len) {
  if (!shape || !len || batch < 1 || n_xcd < 1 || n_xcd > dev::MAX_XCD || n_workers < n_xcd) return FLEET_EINVAL;
  int rc = check_shape(*shape);
  if (rc) return rc;
  if (batch > shape->max_batch) return FLEET_EINVAL;
  const int fma_max = (shape->flags & FLEET_FLAG_PACKED_ONLY) ? 0 : fma_max_from_env();
  return copy_words(build_decode_graph(*shape, batch, n_xcd, n_workers, false, fma_max).serialize(), buf, len);
}

int fleet_graph_dump(fleet_t* f, int32_t batch, void* buf, size_t* len) {
  if (!f || !len || batch < 1 || batch > f->shape.max_batch) return FLEET_EINVAL;
  DevGraph* dg = pick_graph(f, batch, false);
  if (!dg) return FLEET_EINVAL;
  return copy_words(dg->g.serialize(), buf, len);
}

int fleet_trace_read(fleet_t* f, void* buf, size_t* len) {
  if (!f || !len) return FLEET_EINVAL;
  if (!f->trace) return FLEET_EINVAL;
  HIP_TRY(hipDeviceSynchronize());
  const size_t per = (size_t)TRACE_CAP * 8, nw = f->info.n_cu;
  std::vector<int32_t> all(per * nw + nw);
  HIP_TRY(hipMemcpy(all.data(), f->trace, all.size() * 4, hipMemcpyDeviceToHost));
  std::vector<int32_t> out;
  for (size_t w = 0; w < nw; ++w) {
    const int cnt = std::min<int>(std::max(all[per * nw + w], 0), TRACE_CAP);
    out.insert(out.end(), &all[w * per], &all[w * per] + (size_t)cnt * 8);
  }
  int32_t t0 = 0x7fffffff;
  for (size_t i = 0; i < out.size(); i += 8) t0 = std::min(t0, out[i + 6]);
  const bool timing = !(f->shape.flags & FLEET_FLAG_TRACE);   // words 4, 5 are times too
  for (size_t i = 0; i < out.size(); i += 8) {
    out[i + 3] -= t0; out[i + 6] -= t0; out[i + 7] -= t0;
    if (timing) { out[i + 4] -= t0; out[i + 5] -= t0; }
  }
  return copy_words(out, buf, len);
}

int fleet_gemm(int32_t B, int32_t K, int32_t N, const void* x, const void* const* w_copies, int32_t n_copies, float* y,
               int32_t sched_mode, int32_t tile_m, int32_t flags, int32_t reps, void* stream, float* elapsed_ms) {
  if (B < 1 || B > MAX_BATCH || K < 32 || K % 32 || N < 16 || N % 16 || !x || !w_copies || n_copies < 1 || !y || reps < 1 || reps > dev::ECACHE)
    return FLEET_EINVAL;
  if ((int64_t)N * K * 2 >= (int64_t)1 << 31) return FLEET_EINVAL;   // 32-bit byte offsets inside a matrix
  if (sched_mode < FLEET_SCHED_COOPERATIVE || sched_mode > FLEET_SCHED_MSPLIT) return FLEET_EINVAL;
  if (tile_m != 0 && tile_m != 16 && tile_m != 32 && tile_m != 64) return FLEET_EINVAL;
  for (int i = 0; i < n_copies; ++i) if (!w_copies[i]) return FLEET_EINVAL;
  DevInfo info;
  int rc = probe_device(&info, nullptr, 0);
  if (rc) return rc;
  DevGraph dg;
  dg.g = build_gemm_graph(B, K, N, sched_mode, tile_m, flags, reps, n_copies, info.n_xcd, info.n_cu, fma_max_from_env());
  // the MFMA kernels read operand blocks: pack the caller's matrices into private copies
  const bool mfma = dg.g.header[H_PATH] == P_MFMA;
  std::vector<void*> packed;
  void* xp = nullptr;
  int32_t* status = nullptr;
  uint32_t* ctr = nullptr;
  float* gpart = nullptr;   // partial sums of split-K tiles
  auto free_all = [&]() {
    for (void* p : packed) if (p) (void)hipFree(p);
    for (void* p : {(void*)xp, (void*)status, (void*)ctr, (void*)gpart}) if (p) (void)hipFree(p);
  };
  if (mfma) {
    packed.assign(n_copies, nullptr);
    for (int i = 0; i < n_copies; ++i)
      if ((rc = pack_matrix(&packed[i], w_copies[i], N, K, true))) { free_all(); return rc; }
    if ((rc = pack_matrix(&xp, x, B, K, false))) { free_all(); return rc; }
    if (hipDeviceSynchronize() != hipSuccess) { free_all(); return FLEET_EHIP; }
  }
  if ((rc = upload_graph(&dg, nullptr, mfma ? (const void* const*)packed.data() : w_copies, info.n_xcd))) { free_all(); return rc; }
  if ((rc = upload(&status, nullptr, dev::ST_WORDS * 4))) { free_all(); return rc; }
  if ((rc = upload(&ctr, nullptr, (size_t)dg.ctr_words * 4))) { free_all(); return rc; }
  // one region of partial sums: 8 k-slices of the batch padded to whole tiles; one region
  // per XCD under the XCD-aware schedules
  const size_t gpart_bytes = (size_t)8 * ((B + MAX_TILE_ROWS - 1) / MAX_TILE_ROWS * MAX_TILE_ROWS) * N * 4;
  if ((rc = upload(&gpart, nullptr, gpart_bytes * (sched_mode == FLEET_SCHED_UNAWARE ? 1 : dev::MAX_XCD)))) { free_all(); return rc; }
  dev::Params P;
  memset(&P, 0, sizeof(P));
  fill_graph_params(P, &dg);
  P.ctr = ctr;
  P.buf[BUF_GEMM_X] = mfma ? xp : (void*)x; P.buf[BUF_GEMM_Y] = y; P.buf[BUF_GPART] = gpart;
  P.gpart_xcd_bytes = sched_mode == FLEET_SCHED_UNAWARE ? 0 : (int32_t)gpart_bytes;
  P.n_iter = 1;
  P.status = status; P.timeout_ticks = timeout_ticks_from_env(); P.n_xcd = info.n_xcd; P.flags = flags;
  P.batch = B; P.hidden = K;
  const int nm = n_marks(0);
  for (int xc = 0; xc < info.n_xcd; ++xc) { P.q_begin[xc] = dg.g.marks[(size_t)xc * nm + 0]; P.q_end[xc] = dg.g.marks[(size_t)xc * nm + nm - 1]; }
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t he = hipEventCreate(&e0);
  if (he == hipSuccess) he = hipEventCreate(&e1);
  if (he == hipSuccess) {
    const int words = dg.ctr_words;
    hipLaunchKernelGGL(fleet_reset_kernel, dim3((words + 255) / 256), dim3(256), 0, st, ctr, words, -1, 0u, status, 0, 1, 0, -1);
    (void)hipEventRecord(e0, st);
    int lrc = launch_persistent(&dg, P, info.n_cu, st);
    (void)hipEventRecord(e1, st);
    if (lrc) he = hipErrorLaunchFailure;
    if (he == hipSuccess) he = hipEventSynchronize(e1);
    if (he == hipSuccess && elapsed_ms) he = hipEventElapsedTime(elapsed_ms, e0, e1);
  }
  int32_t code[dev::ST_WORDS] = {0};
  if (he == hipSuccess) he = hipMemcpy(code, status, sizeof(code), hipMemcpyDeviceToHost);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  free_all();
  if (he != hipSuccess) { g_last_hip = (int)he; return FLEET_EHIP; }
  return code[dev::ST_CODE];
}

int fleet_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || bytes % 16) return FLEET_EINVAL;
  hipLaunchKernelGGL(fleet_copy_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, bytes / 16);
  HIP_TRY(hipGetLastError());
  return FLEET_OK;
}

// Closed forms: a non-positive divisor is a caller error and gives -1 (0.0 for the model).
int64_t fleet_weight_bytes(int32_t K, int32_t N) { return (int64_t)K * N * 2; }
int64_t fleet_weight_bytes_per_xcd(int32_t K, int32_t N, int32_t n_xcd) {
  return n_xcd > 0 ? (int64_t)K * N * 2 / n_xcd : -1;
}
int64_t fleet_l2_window_bytes(int32_t N, int32_t n_xcd, int32_t tile_n, int32_t tile_k) {
  // one K-chunk of every N-tile of a chiplet's partition (Table "weight sizes")
  if (n_xcd <= 0 || tile_n <= 0) return -1;
  return (int64_t)(N / n_xcd / tile_n) * tile_n * tile_k * 2;
}
double fleet_l2_hit_model(int32_t batch, int32_t tile_m, int32_t workers_per_xcd) {
  if (batch < 1 || tile_m < 0 || workers_per_xcd < 1) return 0.0;
  if (tile_m == 0) tile_m = std::min(MAX_TILE_ROWS, (batch + 15) / 16 * 16);   // whole-batch tile, as in the shape
  const int m_tiles = (batch + tile_m - 1) / tile_m;
  const int R = std::min(workers_per_xcd, m_tiles);
  return R > 0 ? (double)(R - 1) / R : 0.0;
}
double fleet_effective_intensity(int32_t batch, double l2_hit) {
  return l2_hit < 1.0 ? (double)batch / (1.0 - l2_hit) : 0.0;
}
int64_t fleet_step_bytes(const fleet_shape_t* s, int32_t batch, const int32_t* positions) {
  if (!s || !positions) return -1;
  const int64_t H = s->hidden, F = s->ffn, hd = s->head_dim;
  const int64_t per_layer = ((int64_t)(s->n_q_heads + 2 * s->n_kv_heads) * hd * H + (int64_t)s->n_q_heads * hd * H +
                             2 * F * H + F * H) * 2;
  int64_t bytes = per_layer * s->n_layers + (int64_t)s->vocab * H * 2;
  for (int b = 0; b < batch; ++b)   // K and V of every attended slot, all kv heads, all layers
    bytes += (int64_t)s->n_layers * 2 * s->n_kv_heads * hd * 2 * ((int64_t)positions[b] + 1);
  return bytes;
}

}  // extern "C"
