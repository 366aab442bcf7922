// Host side of the C ABI declared in include/fleet.h: device probing, scratch
// allocation, graph upload and the per-step launch of the persistent kernel.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <vector>

#include "../../include/fleet.h"
#include "graph.hpp"
#include "kernels.hip.inc"

namespace {

using namespace fleetg;

constexpr size_t LDS_BYTES = 128 * 1024;  // > half of a CU's 160 KB: one worker per CU
constexpr int TRACE_CAP = 2048;           // records per worker

struct DevInfo {
  int n_cu = 0, n_xcd = 0;
  int per_xcd[dev::MAX_XCD] = {0};
};

struct DevGraph {
  Graph g;
  int32_t *ops = nullptr, *tasks = nullptr, *events = nullptr, *qoff = nullptr, *qents = nullptr;
  int32_t* fat = nullptr;   // [n_tasks][FAT_WORDS]: task words, op words, weight pointers, id
  uint32_t* ctr = nullptr;
  int ctr_words = 0, gcnt_base = 0;
  // memo of wait_event_range for the last queue slice launched
  int memo_begin[dev::MAX_XCD] = {-1, -1, -1, -1, -1, -1, -1, -1}, memo_end[dev::MAX_XCD] = {0}, memo_first = 0, memo_last = -1;
  ~DevGraph() {
    for (void* p : {(void*)ops, (void*)tasks, (void*)events, (void*)qoff, (void*)qents, (void*)fat, (void*)ctr})
      if (p) (void)hipFree(p);
  }
};

int g_last_hip = 0;
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
// range of events that tasks of the launched queue slices wait for (stages of the slices)
void wait_event_range(const Graph& g, dev::Params& P, int n_xcd) {
  int lo = 1 << 30, hi = -1;
  std::vector<char> stage_in;
  for (int x = 0; x < n_xcd; ++x)
    for (int qi = P.q_begin[x]; qi < P.q_end[x]; ++qi) {
      const int32_t* e = &g.qents[((size_t)g.qoff[x] + qi) * QENT_WORDS];
      for (int t = e[Q_FIRST]; t < e[Q_FIRST] + e[Q_COUNT]; ++t) {
        const int w = g.tasks[(size_t)t * TASK_WORDS + T_WAIT_EVENT];
        if (w >= 0) { lo = std::min(lo, w); hi = std::max(hi, w); }
      }
    }
  P.first_wait_event = hi >= 0 ? lo : 0;
  P.last_wait_event = hi;
}

int launch_persistent(DevGraph* dg, dev::Params& P, int n_cu, hipStream_t st) {
  const Graph& g = dg->g;
  const int v = variant_for(g.header[H_PATH], g.header[H_BATCH], g.header[H_TILE_M]);
  const int nx = g.header[H_N_XCD];
  bool same = true;
  for (int x = 0; x < nx; ++x) same = same && dg->memo_begin[x] == P.q_begin[x] && dg->memo_end[x] == P.q_end[x];
  if (!same) {
    wait_event_range(g, P, nx);
    for (int x = 0; x < nx; ++x) { dg->memo_begin[x] = P.q_begin[x]; dg->memo_end[x] = P.q_end[x]; }
    dg->memo_first = P.first_wait_event; dg->memo_last = P.last_wait_event;
  } else {
    P.first_wait_event = dg->memo_first; P.last_wait_event = dg->memo_last;
  }
  void* args[] = {(void*)&P};
  HIP_TRY(hipLaunchKernel(kernel_variant(v, P.page_size > 0), dim3(n_cu), dim3(dev::WG), args, LDS_BYTES, st));
  return FLEET_OK;
}

int prepare_kernel() {
  static bool done = false;
  if (done) return FLEET_OK;
  int dev_id = 0, lds = 0;
  HIP_TRY(hipGetDevice(&dev_id));
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
  done = true;
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

}  // namespace

struct fleet {
  fleet_shape_t shape;
  std::vector<const void*> ln1, wqkv, q_norm, k_norm, wo, ln2, wgu, wdown;
  const void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
  // library-owned copies of the GEMM weights in the operand-block layout of the MFMA
  // kernels (made by fleet_create when max_batch reaches those kernels)
  std::vector<void*> pk_qkv, pk_o, pk_gu, pk_down;
  void* pk_lm = nullptr;
  DevInfo info;
  // scratch activations (device)
  float* x = nullptr; void* n = nullptr; float* qkv = nullptr; void* att = nullptr; void* h = nullptr;
  float* part = nullptr; float* gpart = nullptr; float* gu32 = nullptr; float2* rope = nullptr;
  size_t gpart_bytes = 0;   // bytes of one region of gpart
  int32_t* status = nullptr; int32_t* trace = nullptr;
  std::map<int, std::unique_ptr<DevGraph>> graphs;        // by batch size
  std::map<int, std::unique_ptr<DevGraph>> graphs_loop;   // with the next-token stage (multi-step launches)
  long long timeout_ticks = 0;
  int last_code = 0;
  DevGraph* last_graph = nullptr;
};

namespace {

const void* resolve_weight(const fleet* f, int wkind, int layer, const void* const* gemm_copies, const void** second,
                           bool packed = false) {
  *second = nullptr;
  if (packed && f) {
    switch (wkind) {
      case W_QKV: return f->pk_qkv[layer];
      case W_O: return f->pk_o[layer];
      case W_GU: return f->pk_gu[layer];
      case W_DOWN: return f->pk_down[layer];
      case W_LM: return f->pk_lm;
      default: break;
    }
  }
  switch (wkind) {
    case W_QKV: return f->wqkv[layer];
    case W_O: return f->wo[layer];
    case W_GU: return f->wgu[layer];
    case W_DOWN: return f->wdown[layer];
    case W_LM: return f->lm_head;
    case W_LN1: return f->ln1[layer];
    case W_LN2: return f->ln2[layer];
    case W_FINAL: return f->final_norm;
    case W_EMBED: *second = f->embed; return nullptr;
    case W_GEMM_COPY: return gemm_copies ? gemm_copies[layer] : nullptr;
    default: return nullptr;
  }
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
    const void* second = nullptr;
    w[i] = f || gemm_copies ? resolve_weight(f, o[O_WKIND], o[O_LAYER], gemm_copies, &second, o[O_PATH] == P_MFMA) : nullptr;
    if (o[O_BODY] == B_GEMM && (o[O_AUX2] & 0xff) != W_NONE && f) {   // gain of the fused RMSNorm
      const void* unused = nullptr;
      second = resolve_weight(f, o[O_AUX2] & 0xff, o[O_LAYER], nullptr, &unused);
    }
    w2[i] = second;
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
      if (e[Q_DIST] != D_XCD_RR) continue;
      for (int t = e[Q_FIRST]; t < e[Q_FIRST] + e[Q_COUNT]; ++t) fat[(size_t)t * dev::FAT_WORDS + dev::FAT_GROUP] = e[Q_COUNT];
    }
  if ((rc = upload(&dg->fat, fat.data(), fat.size() * 4))) return rc;
  // G[e], L[x][e], then one arrival counter per (sequence, kv head) for the split-KV merge
  // and one relay word per worker on its own cache line
  // (MFMA graphs: then the arrival counters of split-K GEMM tiles)
  // (then one copy of the device counters per XCD, rows on their own cache lines)
  dg->gcnt_base = dev::C_EVENTS + g.n_events() * (1 + n_xcd) + dev::N_PAIR + n_xcd * dev::RELAY_SLOTS * dev::RELAY_STRIDE +
                  dev::COPY_GROUPS * n_xcd * ((g.n_events() + 31) & ~31);
  dg->ctr_words = dg->gcnt_base + (g.header[H_PATH] == P_MFMA ? dev::GEMM_CNT_WORDS : 0);
  if ((rc = upload(&dg->ctr, nullptr, (size_t)dg->ctr_words * 4))) return rc;
  return FLEET_OK;
}

// reset counters, then run queue slice [q_begin, q_end) of every XCD
int launch(dev::Params& P, DevGraph* dg, int n_cu, int preset_event, hipStream_t st) {
  const int words = dg->ctr_words;
  int preset_word = -1;
  uint32_t preset_val = 0;
  if (preset_event >= 0) {
    preset_word = dev::C_EVENTS + preset_event;
    preset_val = 0x40000000u;   // satisfied whatever the threshold
  }
  const int nE = dg->g.n_events(), nx = dg->g.header[H_N_XCD], cstride = (nE + 31) & ~31;
  const int cbase = dev::C_EVENTS + nE * (1 + nx) + dev::N_PAIR + nx * dev::RELAY_SLOTS * dev::RELAY_STRIDE;
  hipLaunchKernelGGL(fleet_reset_kernel, dim3((words + 255) / 256), dim3(256), 0, st, dg->ctr, words, preset_word,
                     preset_val, P.status, cbase, cstride, dev::COPY_GROUPS * nx, preset_event);
  return launch_persistent(dg, P, n_cu, st);
}

void fill_graph_params(dev::Params& P, const DevGraph* dg) {
  P.ops = dg->ops; P.tasks = dg->tasks; P.events = dg->events; P.qoff = dg->qoff; P.qents = dg->qents;
  P.fat = dg->fat; P.ctr = dg->ctr; P.n_events = dg->g.n_events(); P.gcnt_base = dg->gcnt_base;
}

int get_graph(fleet* f, int batch, DevGraph** out, bool loop = false) {
  auto& cache = loop ? f->graphs_loop : f->graphs;
  auto it = cache.find(batch);
  if (it != cache.end()) { *out = it->second.get(); return FLEET_OK; }
  std::unique_ptr<DevGraph> dg(new (std::nothrow) DevGraph());
  if (!dg) return FLEET_ENOMEM;
  dg->g = build_decode_graph(f->shape, batch, f->info.n_xcd, f->info.n_cu, loop);
  int rc = upload_graph(dg.get(), f, nullptr, f->info.n_xcd);
  if (rc) return rc;
  *out = dg.get();
  cache[batch] = std::move(dg);
  return FLEET_OK;
}
struct KvPaging {   // paged KV cache: k_cache / v_cache are page pools
  const int32_t* table = nullptr;   // device [batch][stride] page indices
  int page_size = 0, n_pages = 0, stride = 0;
};

// n_tokens > 0: the whole step n_tokens times in one launch (graph with the next-token stage)
int run_layers(fleet* f, int batch, int layer_begin, int layer_end, bool with_ingest, bool with_final,
               const void* hidden_in, const int32_t* tokens, void* k_cache, void* v_cache, const int32_t* positions,
               float* hidden_out, float* logits, hipStream_t st, int n_tokens = 0, int32_t* tokens_out = nullptr,
               const KvPaging* paging = nullptr) {
  // the kernels move activations, cache rows and logits in 16-byte pieces
  for (const void* p : {hidden_in, (const void*)k_cache, (const void*)v_cache, (const void*)hidden_out, (const void*)logits})
    if ((uintptr_t)p % 16 != 0) return FLEET_EINVAL;
  for (const void* p : {(const void*)tokens, (const void*)positions, (const void*)tokens_out, paging ? (const void*)paging->table : nullptr})
    if ((uintptr_t)p % 4 != 0) return FLEET_EINVAL;
  DevGraph* dg = nullptr;
  int rc = get_graph(f, batch, &dg, n_tokens > 0);
  if (rc) return rc;
  const Graph& g = dg->g;
  const int L = f->shape.n_layers, n_marks = L + 3, nx = f->info.n_xcd;
  dev::Params P;
  memset(&P, 0, sizeof(P));
  fill_graph_params(P, dg);
  P.buf[BUF_X] = f->x; P.buf[BUF_N] = f->n; P.buf[BUF_QKV] = f->qkv; P.buf[BUF_ATT] = f->att; P.buf[BUF_H] = f->h;
  P.buf[BUF_PART] = f->part; P.buf[BUF_GPART] = f->gpart; P.buf[BUF_GU32] = f->gu32; P.buf[BUF_HIDDEN_IN] = (void*)hidden_in; P.buf[BUF_TOKENS] = (void*)tokens;
  P.buf[BUF_KC] = k_cache; P.buf[BUF_VC] = v_cache; P.buf[BUF_POS] = (void*)positions;
  P.buf[BUF_HIDDEN_OUT] = hidden_out; P.buf[BUF_LOGITS] = logits; P.buf[BUF_TOKENS_OUT] = tokens_out;
  P.n_iter = n_tokens > 0 ? n_tokens : 1;
  P.gpart_xcd_bytes = f->shape.sched_mode == FLEET_SCHED_UNAWARE ? 0 : (int32_t)f->gpart_bytes;
  if (paging) {
    P.buf[BUF_PT] = (void*)paging->table;
    P.page_size = paging->page_size; P.n_pages = paging->n_pages; P.pt_stride = paging->stride;
  }
  P.status = f->status; P.trace_cap = TRACE_CAP;
  // (no trace of a multi-step launch: the record area holds one step)
  P.trace = (n_tokens == 0 && (f->shape.flags & (FLEET_FLAG_TRACE | FLEET_FLAG_TIMING))) ? f->trace : nullptr;
  P.rope = f->rope; P.timeout_ticks = f->timeout_ticks; P.n_xcd = nx; P.flags = f->shape.flags;
  P.nq = f->shape.n_q_heads; P.nkv = f->shape.n_kv_heads; P.hd = f->shape.head_dim; P.max_batch = f->shape.max_batch;
  P.max_seq = f->shape.max_seq; P.hidden = f->shape.hidden; P.ffn = f->shape.ffn; P.batch = batch; P.eps = f->shape.rms_eps; P.vocab = f->shape.vocab;
  const int mb = with_ingest ? 0 : 1 + layer_begin;
  int me = with_final ? L + 2 : 1 + layer_end;
  for (int x = 0; x < nx; ++x) {
    P.q_begin[x] = g.marks[(size_t)x * n_marks + mb];
    P.q_end[x] = g.marks[(size_t)x * n_marks + me];
  }
  // without the final stage and LM head the queue must stop before them; without
  // logits the LM head is skipped by ending at the mark of the final stage + its
  // own entries -- the final stage always runs when requested (it writes hidden_out)
  int preset = with_ingest ? -1 : g.xready[layer_begin];
  f->last_graph = dg;
  return launch(P, dg, f->info.n_cu, preset, st);
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
  std::unique_ptr<fleet> f(new (std::nothrow) fleet());
  if (!f) return FLEET_ENOMEM;
  f->shape = *shape;
  f->ln1.assign(w->ln1, w->ln1 + L); f->wqkv.assign(w->wqkv, w->wqkv + L); f->q_norm.assign(w->q_norm, w->q_norm + L);
  f->k_norm.assign(w->k_norm, w->k_norm + L); f->wo.assign(w->wo, w->wo + L); f->ln2.assign(w->ln2, w->ln2 + L);
  f->wgu.assign(w->wgu, w->wgu + L); f->wdown.assign(w->wdown, w->wdown + L);
  f->embed = w->embed; f->final_norm = w->final_norm; f->lm_head = w->lm_head;
  f->timeout_ticks = timeout_ticks_from_env();
  if ((rc = probe_device(&f->info, nullptr, 0))) return rc;
  for (int x = 0; x < f->info.n_xcd; ++x)
    if (f->info.per_xcd[x] == 0) return FLEET_EDEVICE;

  const size_t mb = shape->max_batch, H = shape->hidden, F = shape->ffn;
  const size_t NQKV = (size_t)(shape->n_q_heads + 2 * shape->n_kv_heads) * shape->head_dim;
  const size_t QD = (size_t)shape->n_q_heads * shape->head_dim;
  const size_t grp = shape->n_q_heads / shape->n_kv_heads;
  if ((rc = upload(&f->x, nullptr, mb * H * 4))) return rc;
  // bf16 activations: feature dimension padded to whole 256-wide chunks (the MFMA kernels
  // store them chunk-tiled)
  // (the MFMA kernels store them as operand blocks of 16 rows)
  auto pad256 = [](size_t k) { return (k + 255) / 256 * 256; };
  const size_t mb16 = (mb + 15) / 16 * 16;
  if ((rc = upload((char**)&f->n, nullptr, mb16 * pad256(H) * 2))) return rc;
  if ((rc = upload(&f->qkv, nullptr, mb * NQKV * 4))) return rc;
  if ((rc = upload((char**)&f->att, nullptr, mb16 * pad256(QD) * 2))) return rc;
  if ((rc = upload((char**)&f->h, nullptr, mb16 * pad256(F) * 2))) return rc;
  if ((rc = upload(&f->part, nullptr, mb * shape->n_kv_heads * 32 * grp * dev::PART_STRIDE * 4))) return rc;
  if (shape->max_batch > fma_max_batch()) {
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
  // partial sums of split-K GEMM tiles (MFMA kernels): up to 8 k-slices of the widest output a
  // split plan can have, batch rows padded to the 64 one m-tile can hold
  if (shape->max_batch > fma_max_batch()) {
    size_t nmax = std::max({NQKV, H, 2 * F});
    if (shape->vocab > 0 && (size_t)shape->vocab / 16 * 4 <= (size_t)GEMM_TILE_COUNTERS) nmax = std::max(nmax, (size_t)shape->vocab);
    // (a region per XCD under the XCD-aware schedules)
    f->gpart_bytes = 8 * 64 * nmax * 4;
    if ((rc = upload(&f->gpart, nullptr, f->gpart_bytes * (shape->sched_mode == FLEET_SCHED_UNAWARE ? 1 : dev::MAX_XCD)))) return rc;
  }
  if (shape->flags & FLEET_FLAG_UNFUSED_SILU)   // fp32 [gate | up] sums of the unfused gate|up GEMM
    if ((rc = upload(&f->gu32, nullptr, mb * 2 * F * 4))) return rc;
  if ((rc = upload(&f->status, nullptr, dev::ST_WORDS * 4))) return rc;
  HIP_TRY(hipMemset(f->status, 0, dev::ST_WORDS * 4));
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
  for (void* p : {(void*)f->x, f->n, (void*)f->qkv, f->att, f->h, (void*)f->part, (void*)f->gpart, (void*)f->gu32, (void*)f->rope, (void*)f->status, (void*)f->trace})
    if (p) (void)hipFree(p);
  for (auto* v : {&f->pk_qkv, &f->pk_o, &f->pk_gu, &f->pk_down})
    for (void* p : *v) if (p) (void)hipFree(p);
  if (f->pk_lm) (void)hipFree(f->pk_lm);
  delete f;
  return FLEET_OK;
}

int fleet_decode_step(fleet_t* f, int32_t batch, const void* hidden_in, const int32_t* tokens, void* k_cache,
                      void* v_cache, const int32_t* positions, float* hidden_out, float* logits, void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !k_cache || !v_cache || !positions || !hidden_out) return FLEET_EINVAL;
  if (!hidden_in && !(tokens && f->embed)) return FLEET_EINVAL;
  if (!logits && f->shape.vocab > 0) {
    // the LM head is part of the step; callers that do not want logits run layers only
    return FLEET_EINVAL;
  }
  return run_layers(f, batch, 0, f->shape.n_layers, true, true, hidden_in, tokens, k_cache, v_cache, positions,
                    hidden_out, logits, (hipStream_t)stream);
}

int fleet_decode_layers(fleet_t* f, int32_t batch, int32_t layer_begin, int32_t layer_end, const float* x_in,
                        void* k_cache, void* v_cache, const int32_t* positions, float* x_out, float* logits,
                        void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !k_cache || !v_cache || !positions || !x_in || !x_out) return FLEET_EINVAL;
  const int L = f->shape.n_layers;
  if (layer_begin < 0 || layer_end > L || layer_begin >= layer_end) return FLEET_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const size_t bytes = (size_t)batch * f->shape.hidden * 4;
  HIP_TRY(hipMemcpyAsync(f->x, x_in, bytes, hipMemcpyDeviceToDevice, st));
  const bool fin = layer_end == L && logits && f->shape.vocab > 0;
  int rc = run_layers(f, batch, layer_begin, layer_end, false, fin, nullptr, nullptr, k_cache, v_cache, positions,
                      x_out, logits, st);
  if (rc) return rc;
  if (!fin) HIP_TRY(hipMemcpyAsync(x_out, f->x, bytes, hipMemcpyDeviceToDevice, st));
  return FLEET_OK;
}

int fleet_decode_step_paged(fleet_t* f, int32_t batch, const void* hidden_in, const int32_t* tokens, void* k_pool,
                            void* v_pool, const int32_t* page_table, int32_t page_size, int32_t n_pages,
                            int32_t table_stride, const int32_t* positions, float* hidden_out, float* logits,
                            void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !k_pool || !v_pool || !positions || !hidden_out || !page_table)
    return FLEET_EINVAL;
  if (!hidden_in && !(tokens && f->embed)) return FLEET_EINVAL;
  if (!logits && f->shape.vocab > 0) return FLEET_EINVAL;   // the LM head is part of the step
  if (page_size < 64 || (page_size & (page_size - 1)) || n_pages < 1 || table_stride < 1) return FLEET_EINVAL;
  // the kernel addresses a page with 32-bit page arithmetic inside one layer's pool
  if ((int64_t)n_pages * f->shape.n_kv_heads * page_size > (int64_t)1 << 40) return FLEET_EINVAL;
  KvPaging pg;
  pg.table = page_table; pg.page_size = page_size; pg.n_pages = n_pages; pg.stride = table_stride;
  return run_layers(f, batch, 0, f->shape.n_layers, true, true, hidden_in, tokens, k_pool, v_pool, positions, hidden_out,
                    logits, (hipStream_t)stream, 0, nullptr, &pg);
}

int fleet_decode_tokens(fleet_t* f, int32_t batch, int32_t* tokens, void* k_cache, void* v_cache, int32_t* positions,
                        int32_t n_tokens, int32_t* tokens_out, float* hidden_out, float* logits, void* stream) {
  if (!f || batch < 1 || batch > f->shape.max_batch || !tokens || !k_cache || !v_cache || !positions || !tokens_out ||
      !hidden_out || !logits || n_tokens < 1 || n_tokens > 65536)
    return FLEET_EINVAL;
  if (f->shape.vocab <= 0 || !f->embed || !f->lm_head || !f->final_norm) return FLEET_EINVAL;
  return run_layers(f, batch, 0, f->shape.n_layers, true, true, nullptr, tokens, k_cache, v_cache, positions, hidden_out,
                    logits, (hipStream_t)stream, n_tokens, tokens_out);
}

int fleet_last_status(fleet_t* f, fleet_status_t* out) {
  if (!f || !out) return FLEET_EINVAL;
  memset(out, 0, sizeof(*out));
  hipError_t e = hipDeviceSynchronize();
  out->hip_error = e != hipSuccess ? (int)e : g_last_hip;
  int32_t st[dev::ST_WORDS];
  HIP_TRY(hipMemcpy(st, f->status, sizeof(st), hipMemcpyDeviceToHost));
  out->code = e != hipSuccess ? FLEET_EHIP : st[dev::ST_CODE];
  out->task = st[dev::ST_TASK]; out->event = st[dev::ST_EVENT];
  out->observed = st[dev::ST_OBSERVED]; out->needed = st[dev::ST_NEEDED];
  out->n_xcd = f->info.n_xcd;
  for (int x = 0; x < 8; ++x) out->workers[x] = st[dev::ST_WORKERS + x];
  return FLEET_OK;
}

int fleet_graph_build(const fleet_shape_t* shape, int32_t batch, int32_t n_xcd, int32_t n_workers, void* buf, size_t* len) {
  if (!shape || !len || batch < 1 || n_xcd < 1 || n_xcd > dev::MAX_XCD || n_workers < n_xcd) return FLEET_EINVAL;
  int rc = check_shape(*shape);
  if (rc) return rc;
  if (batch > shape->max_batch) return FLEET_EINVAL;
  std::vector<int32_t> words = build_decode_graph(*shape, batch, n_xcd, n_workers).serialize();
  const size_t need = words.size() * 4;
  if (!buf || *len < need) { *len = need; return buf ? FLEET_ESMALL : FLEET_OK; }
  memcpy(buf, words.data(), need);
  *len = need;
  return FLEET_OK;
}

int fleet_graph_dump(fleet_t* f, int32_t batch, void* buf, size_t* len) {
  if (!f || !len || batch < 1 || batch > f->shape.max_batch) return FLEET_EINVAL;
  DevGraph* dg = nullptr;
  int rc = get_graph(f, batch, &dg);
  if (rc) return rc;
  std::vector<int32_t> words = dg->g.serialize();
  const size_t need = words.size() * 4;
  if (!buf || *len < need) { *len = need; return buf ? FLEET_ESMALL : FLEET_OK; }
  memcpy(buf, words.data(), need);
  *len = need;
  return FLEET_OK;
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
  const size_t need = out.size() * 4;
  if (!buf || *len < need) { *len = need; return buf ? FLEET_ESMALL : FLEET_OK; }
  memcpy(buf, out.data(), need);
  *len = need;
  return FLEET_OK;
}

int fleet_gemm(int32_t B, int32_t K, int32_t N, const void* x, const void* const* w_copies, int32_t n_copies, float* y,
               int32_t sched_mode, int32_t tile_m, int32_t flags, int32_t reps, void* stream, float* elapsed_ms) {
  if (B < 1 || B > 64 || K < 32 || K % 32 || N < 16 || N % 16 || !x || !w_copies || n_copies < 1 || !y || reps < 1 || reps > 4096)
    return FLEET_EINVAL;
  if (sched_mode < FLEET_SCHED_COOPERATIVE || sched_mode > FLEET_SCHED_MSPLIT) return FLEET_EINVAL;
  if (tile_m != 0 && tile_m != 16 && tile_m != 32 && tile_m != 64) return FLEET_EINVAL;
  for (int i = 0; i < n_copies; ++i) if (!w_copies[i]) return FLEET_EINVAL;
  DevInfo info;
  int rc = probe_device(&info, nullptr, 0);
  if (rc) return rc;
  DevGraph dg;
  dg.g = build_gemm_graph(B, K, N, sched_mode, tile_m, flags, reps, n_copies, info.n_xcd, info.n_cu);
  // the MFMA kernels read operand blocks: pack the caller's matrices into private copies
  const bool mfma = dg.g.header[H_PATH] == P_MFMA;
  std::vector<void*> packed;
  void* xp = nullptr;
  auto free_packed = [&]() { for (void* p : packed) if (p) (void)hipFree(p); if (xp) (void)hipFree(xp); };
  if (mfma) {
    packed.assign(n_copies, nullptr);
    for (int i = 0; i < n_copies; ++i)
      if ((rc = pack_matrix(&packed[i], w_copies[i], N, K, true))) { free_packed(); return rc; }
    if ((rc = pack_matrix(&xp, x, B, K, false))) { free_packed(); return rc; }
    if (hipDeviceSynchronize() != hipSuccess) { free_packed(); return FLEET_EHIP; }
  }
  if ((rc = upload_graph(&dg, nullptr, mfma ? (const void* const*)packed.data() : w_copies, info.n_xcd))) { free_packed(); return rc; }
  int32_t* status = nullptr;
  if ((rc = upload(&status, nullptr, dev::ST_WORDS * 4))) { free_packed(); return rc; }
  float* gpart = nullptr;   // partial sums of split-K tiles
  const size_t gpart_bytes = (size_t)8 * 64 * N * 4;   // one region; one per XCD under the XCD-aware schedules
  if ((rc = upload(&gpart, nullptr, gpart_bytes * (sched_mode == FLEET_SCHED_UNAWARE ? 1 : dev::MAX_XCD)))) { (void)hipFree(status); free_packed(); return rc; }
  dev::Params P;
  memset(&P, 0, sizeof(P));
  fill_graph_params(P, &dg);
  P.buf[BUF_GEMM_X] = mfma ? xp : (void*)x; P.buf[BUF_GEMM_Y] = y; P.buf[BUF_GPART] = gpart;
  P.gpart_xcd_bytes = sched_mode == FLEET_SCHED_UNAWARE ? 0 : (int32_t)gpart_bytes;
  P.n_iter = 1;
  P.status = status; P.timeout_ticks = timeout_ticks_from_env(); P.n_xcd = info.n_xcd; P.flags = flags;
  P.batch = B; P.hidden = K;
  for (int xc = 0; xc < info.n_xcd; ++xc) { P.q_begin[xc] = dg.g.marks[(size_t)xc * 3 + 0]; P.q_end[xc] = dg.g.marks[(size_t)xc * 3 + 2]; }
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t he = hipEventCreate(&e0);
  if (he == hipSuccess) he = hipEventCreate(&e1);
  if (he == hipSuccess) {
    const int words = dg.ctr_words;
    hipLaunchKernelGGL(fleet_reset_kernel, dim3((words + 255) / 256), dim3(256), 0, st, dg.ctr, words, -1, 0u, status, 0, 1, 0, -1);
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
  (void)hipFree(status);
  (void)hipFree(gpart);
  free_packed();
  if (he != hipSuccess) { g_last_hip = (int)he; return FLEET_EHIP; }
  return code[dev::ST_CODE];
}

int fleet_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || bytes % 16) return FLEET_EINVAL;
  hipLaunchKernelGGL(fleet_copy_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, bytes / 16);
  HIP_TRY(hipGetLastError());
  return FLEET_OK;
}

int64_t fleet_weight_bytes(int32_t K, int32_t N) { return (int64_t)K * N * 2; }
int64_t fleet_weight_bytes_per_xcd(int32_t K, int32_t N, int32_t n_xcd) { return (int64_t)K * N * 2 / n_xcd; }
int64_t fleet_l2_window_bytes(int32_t N, int32_t n_xcd, int32_t tile_n, int32_t tile_k) {
  // one K-chunk of every N-tile of a chiplet's partition (Table "weight sizes")
  return (int64_t)(N / n_xcd / tile_n) * tile_n * tile_k * 2;
}
double fleet_l2_hit_model(int32_t batch, int32_t tile_m, int32_t workers_per_xcd) {
  const int m_tiles = (batch + tile_m - 1) / tile_m;
  const int R = std::min(workers_per_xcd, m_tiles);
  return R > 0 ? (double)(R - 1) / R : 0.0;
}
double fleet_effective_intensity(int32_t batch, double l2_hit) { return (double)batch / (1.0 - l2_hit); }
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
