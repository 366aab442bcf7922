// Host-side task-graph builder (see graph.hpp for the layout and citations).
#include "graph.hpp"

#include <algorithm>
#include <cstring>

namespace fleetg {

// M-split applies to an operator with T >= 2 m-tiles where T divides the XCD count
static bool msplit_applies(int sched, int path, int m_tiles, int n_xcd) {
  return sched == FLEET_SCHED_MSPLIT && path == P_MFMA && m_tiles >= 2 && n_xcd % m_tiles == 0;
}

namespace {

struct Builder {
  Graph g;
  int n_xcd, n_workers, sched, batch;
  std::vector<std::vector<int32_t>> queues;  // per XCD, QENT_WORDS per entry
  int stage = 0;

  Builder(int nx, int nw, int sc, int b) : n_xcd(nx), n_workers(nw), sched(sc), batch(b), queues(nx) {}

  int add_op(Body body, int layer, Epi epi, Path path, int K, int N, int unit_rows, int n_units,
             int m_tiles, int tile_m, Buf in, Buf out, int aux, WKind wk, int aux2 = 0) {
    int32_t w[OP_WORDS] = {0};
    w[O_BODY] = body; w[O_LAYER] = layer; w[O_EPI] = epi; w[O_PATH] = path; w[O_K] = K; w[O_N] = N;
    w[O_UNIT_ROWS] = unit_rows; w[O_N_UNITS] = n_units; w[O_M_TILES] = m_tiles; w[O_TILE_M] = tile_m;
    w[O_IN_BUF] = in; w[O_OUT_BUF] = out; w[O_AUX] = aux; w[O_WKIND] = wk; w[O_BATCH] = batch;
    w[O_AUX2] = aux2;
    g.ops.insert(g.ops.end(), w, w + OP_WORDS);
    return g.n_ops() - 1;
  }
  int add_event(int threshold, EventKind kind, int mask, int n_tasks) {
    int32_t w[EVENT_WORDS] = {threshold, kind, mask, n_tasks};
    g.events.insert(g.events.end(), w, w + EVENT_WORDS);
    return g.n_events() - 1;
  }
  int add_task(int op, Scope scope, int xcd, int a0, int a1, int a2, int a3, int wait_ev, int sig_ev) {
    int32_t w[TASK_WORDS] = {0};
    w[T_OP] = op; w[T_SCOPE] = scope; w[T_XCD] = xcd; w[T_A0] = a0; w[T_A1] = a1; w[T_A2] = a2;
    w[T_A3] = a3; w[T_WAIT_EVENT] = wait_ev; w[T_SIGNAL_EVENT] = sig_ev; w[T_STAGE] = stage;
    g.tasks.insert(g.tasks.end(), w, w + TASK_WORDS);
    return g.n_tasks() - 1;
  }
  void push_q(int xcd, int first, int count, Dist d) {
    int32_t w[QENT_WORDS] = {first, count, d, stage};
    queues[xcd].insert(queues[xcd].end(), w, w + QENT_WORDS);
  }

  // A stage of CU-tasks, one per item; item i belongs to XCD key(i) % n_xcd in
  // the cooperative schedule (round-robin inside the XCD), to any worker in the
  // chiplet-unaware one.  args(i) fills A0..A3.  Returns the signalled event.
  // Few tasks per XCD (at most min_per_xcd on average): each signals the device counter itself
  // (one atomic less on the path).  More: two-level, one device-level signal per XCD.
  // from_top: the XCD's tasks go to its highest ranks (the stage after it leaves those idle).
  template <class KeyF, class ArgF>
  int cu_stage(int op, int n_items, int wait_ev, KeyF key, ArgF args, int min_per_xcd = 1, bool from_top = false) {
    int ev;
    const bool two_level = sched != FLEET_SCHED_UNAWARE && n_items > min_per_xcd * n_xcd;
    if (!two_level) {
      ev = add_event(n_items, EV_DIRECT, 0, n_items);
    } else {   // one device-level signal per XCD that runs some of the tasks
      int mask = 0, nx = 0;
      for (int i = 0; i < n_items; ++i) mask |= 1 << (key(i) % n_xcd);
      for (int x = 0; x < n_xcd; ++x) nx += (mask >> x) & 1;
      ev = add_event(nx, EV_TWO_LEVEL_CU, mask, n_items);
    }
    if (sched == FLEET_SCHED_UNAWARE) {
      int first = g.n_tasks();
      for (int i = 0; i < n_items; ++i) {
        int a[4]; args(i, a);
        add_task(op, S_CU, -1, a[0], a[1], a[2], a[3], wait_ev, ev);
      }
      for (int x = 0; x < n_xcd; ++x) push_q(x, first, n_items, D_DEV_RR);
    } else {
      for (int x = 0; x < n_xcd; ++x) {
        int first = g.n_tasks(), cnt = 0;
        for (int i = 0; i < n_items; ++i) {
          if (key(i) % n_xcd != x) continue;
          int a[4]; args(i, a);
          add_task(op, S_CU, x, a[0], a[1], a[2], a[3], wait_ev, ev);
          ++cnt;
        }
        if (cnt) push_q(x, first, cnt, from_top ? D_XCD_RR_TOP : D_XCD_RR);
      }
    }
    ++stage;
    return ev;
  }

  // One GEMM device-task.  Cooperative: one chiplet-task per XCD over a contiguous
  // slice of the output units (section 3.2, N-split).  Unaware: 2-D tiles
  // (unit group x m-tile) in N-major order, dealt to any worker.
  // skip[x] (cooperative schedule only): the first skip[x] workers of XCD x take no units
  // of this chiplet-task (they are still busy with the stage before it).
  int gemm_stage(int op, int wait_ev, const std::vector<int>* skip = nullptr) {
    const int32_t* o = &g.ops[(size_t)op * OP_WORDS];
    const int U = o[O_N_UNITS], mt = o[O_M_TILES];
    int ev;
    if (sched == FLEET_SCHED_UNAWARE) {
      // FMA path: as many units per CU-task as spread U over the workers once;
      // MFMA path: the operator's tile plan (units per tile, k-slices)
      const bool mfma = o[O_PATH] == P_MFMA;
      const int cu_units = mfma ? std::max(1, (o[O_AUX2] >> 12) & 15) : std::max(1, U / std::max(1, n_workers));
      const int ksn = mfma ? std::max(1, (o[O_AUX2] >> 16) & 15) : 1;
      int ng = (U + cu_units - 1) / cu_units;
      ev = add_event(ng * mt * ksn, EV_DIRECT, 0, ng * mt * ksn);
      int first = g.n_tasks();
      for (int m = 0; m < mt; ++m)
        for (int ks = 0; ks < ksn; ++ks)
          for (int gi = 0; gi < ng; ++gi) {
            int u0 = gi * cu_units, cnt = std::min(cu_units, U - u0);
            add_task(op, S_CU, -1, u0, cnt, m, ks, wait_ev, ev);
          }
      for (int x = 0; x < n_xcd; ++x) push_q(x, first, ng * mt * ksn, D_DEV_RR);
    } else if (msplit_applies(sched, o[O_PATH], mt, n_xcd)) {
      // M-split: XCD x works on m-tile x / xpm only (A3 = m-tile + 1) and on the
      // (x % xpm)-th of xpm slices of the units
      const int xpm = n_xcd / mt;
      int mask = 0, nx = 0;
      for (int x = 0; x < n_xcd; ++x) {
        int part = x % xpm, u0 = (int)((int64_t)U * part / xpm), u1 = (int)((int64_t)U * (part + 1) / xpm);
        if (u1 > u0) { mask |= 1 << x; ++nx; }
      }
      ev = add_event(nx, EV_TWO_LEVEL, mask, nx);
      for (int x = 0; x < n_xcd; ++x) {
        int part = x % xpm, u0 = (int)((int64_t)U * part / xpm), u1 = (int)((int64_t)U * (part + 1) / xpm);
        if (u1 <= u0) continue;
        int t = add_task(op, S_CHIPLET, x, u0, u1 - u0, 0, x / xpm + 1, wait_ev, ev);
        push_q(x, t, 1, D_CHIPLET);
      }
    } else {
      int mask = 0, nx = 0;
      for (int x = 0; x < n_xcd; ++x) {
        int u0 = (int)((int64_t)U * x / n_xcd), u1 = (int)((int64_t)U * (x + 1) / n_xcd);
        if (u1 > u0) { mask |= 1 << x; ++nx; }
      }
      ev = add_event(nx, EV_TWO_LEVEL, mask, nx);
      for (int x = 0; x < n_xcd; ++x) {
        int u0 = (int)((int64_t)U * x / n_xcd), u1 = (int)((int64_t)U * (x + 1) / n_xcd);
        if (u1 <= u0) continue;
        int t = add_task(op, S_CHIPLET, x, u0, u1 - u0, skip ? (*skip)[x] : 0, 0, wait_ev, ev);
        push_q(x, t, 1, D_CHIPLET);
      }
    }
    ++stage;
    return ev;
  }

  void mark_all() {
    for (int x = 0; x < n_xcd; ++x) g.marks.push_back((int32_t)queues[x].size() / QENT_WORDS);
  }

  Graph finish(int n_layers, int tile_m, int path, int n_splits, int m_tiles) {
    g.qoff.assign(n_xcd + 1, 0);
    for (int x = 0; x < n_xcd; ++x) {
      g.qoff[x + 1] = g.qoff[x] + (int32_t)queues[x].size() / QENT_WORDS;
      g.qents.insert(g.qents.end(), queues[x].begin(), queues[x].end());
    }
    // marks were pushed stage-major ([mark][xcd]); store them [xcd][mark]
    int n_marks = n_xcd ? (int)g.marks.size() / n_xcd : 0;
    std::vector<int32_t> m((size_t)n_xcd * n_marks);
    for (int k = 0; k < n_marks; ++k)
      for (int x = 0; x < n_xcd; ++x) m[(size_t)x * n_marks + k] = g.marks[(size_t)k * n_xcd + x];
    g.marks.swap(m);
    g.header.assign(HEADER_WORDS, 0);
    int32_t* h = g.header.data();
    h[H_MAGIC] = MAGIC; h[H_VERSION] = 1; h[H_N_OPS] = g.n_ops(); h[H_N_TASKS] = g.n_tasks();
    h[H_N_EVENTS] = g.n_events(); h[H_N_XCD] = n_xcd; h[H_N_QENT] = g.n_qent(); h[H_N_LAYERS] = n_layers;
    h[H_BATCH] = batch; h[H_SCHED] = sched; h[H_TILE_M] = tile_m; h[H_PATH] = path;
    h[H_N_SPLITS] = n_splits; h[H_N_WORKERS] = n_workers; h[H_M_TILES] = m_tiles;
    h[H_TOTAL_WORDS] = (int32_t)(HEADER_WORDS + g.ops.size() + g.tasks.size() + g.events.size() +
                                 g.qoff.size() + g.qents.size() + g.marks.size() + g.xready.size());
    return std::move(g);
  }
};

}  // namespace

std::vector<int32_t> Graph::serialize() const {
  std::vector<int32_t> out;
  out.reserve(header.size() + ops.size() + tasks.size() + events.size() + qoff.size() + qents.size() +
              marks.size() + xready.size());
  for (const auto* v : {&header, &ops, &tasks, &events, &qoff, &qents, &marks, &xready})
    out.insert(out.end(), v->begin(), v->end());
  return out;
}

int mfma_blocks(int tile_m) { return tile_m <= 16 ? 1 : tile_m <= 32 ? 2 : 4; }

// Tile plan of an MFMA GEMM operator: G units per tile and KS k-slices for the tiles of one
// XCD's unit slice (ux units, m_tiles m-tiles each, wpx workers), by a cost model fitted to
// a sweep of plans on MI355X (integer arithmetic; times in ns, sizes in KB, rates in KB/us):
//   * a worker streams a tile at the rate its bytes in flight allow -- (D - 1) rounds of
//     G * nb row blocks of 8 KB, over a loaded latency of 2.5 us -- capped per CU (30, 45
//     where several m-tiles share the weights through the L2) and by the XCD's share
//     of the memory bandwidth (700 per XCD over the workers that hold a tile, times the number
//     of m-tiles that share a weight read);
//   * a round costs 0.1 us per block of 16 batch rows (activation reads, MFMAs);
//   * a tile costs 1 us on top (pipeline fill, cross-wave reduction, epilogue), a split-K tile
//     3 us + 0.4 us per slice (partial sums out, arrival counter, the last arriver's reduction).
// (The latency and the cost per slice were refitted inside the decode step: with 3.8 us and
// 0.2 us, which the isolated sweep suggested, the down projection at batch 17-32 took 8 units
// x 8 slices where 4 x 4 is 1.4 to 3 % of a step faster.)
// The worker with the most tiles decides (+10 % where the tiles do not divide evenly among
// the workers).  Ties: more units per tile, then fewer slices.
// allow_split = false: one k-slice only.
MfmaPlan plan_mfma(int ux, int wpx, int K, int nb, int mt_blocks, int m_tiles, bool allow_split) {
  const int gmax = std::max(1, ((mt_blocks >= 4 || nb == 2) ? 6 : 8) / nb);
  const int depth = (mt_blocks >= 4 || (mt_blocks == 2 && nb == 1)) ? 3 : 4;   // operand rounds held (kernel: MfmaCfg::D)
  ux = std::max(1, ux); wpx = std::max(1, wpx); m_tiles = std::max(1, m_tiles);
  const bool shared = m_tiles > 1;
  MfmaPlan best{1, 1, 0};
  long best_cost = -1;
  for (int G = 1; G <= std::min(gmax, ux); ++G)
    for (int KS = 1; KS <= 8; KS *= 2) {
      if (KS > 1 && (!allow_split || K % (KS * 256) != 0)) continue;
      const long tiles = (long)((ux + G - 1) / G) * KS * m_tiles;
      const long per_worker = (tiles + wpx - 1) / wpx, active = std::min<long>(tiles, wpx);
      const long kc = K / KS, rounds = (kc + 255) / 256;
      const long inflight_kb = (long)(depth - 1) * G * nb * 8;
      long rate = inflight_kb * 1000 / 2500;
      rate = std::min(rate, shared ? 45L : 30L);
      rate = std::min(rate, 700L * std::min(m_tiles, wpx) / active);
      rate = std::max(rate, 1L);
      const long tile_kb = (long)G * nb * kc / 32;
      const long tile_ns = tile_kb * 1000 / rate + rounds * mt_blocks * 100 + (KS > 1 ? 3000 + 400 * KS : 1000);
      long cost = per_worker * tile_ns;
      if (tiles % wpx != 0) cost += cost / 10;   // idle or unequally loaded workers: measured worse than the rates above say
      if (best_cost < 0 || cost < best_cost || (cost == best_cost && (G > best.G || (G == best.G && KS < best.KS)))) {
        best_cost = cost; best.G = G; best.KS = KS;
      }
    }
  return best;
}

// the plan of an operator with n_units units under the given schedule
static MfmaPlan plan_for(int sched, int flags, int n_units, int K, int nb, int tile_m, int m_tiles, int n_xcd, int n_workers) {
  const bool split_ok = !(flags & FLEET_FLAG_NO_SPLITK) && (long)n_units * m_tiles <= GEMM_TILE_COUNTERS;
  const int wpx = n_workers / std::max(1, n_xcd);
  // Small weight shares (one m-tile, at most RESIDENT_UNITS units per worker, K up to RESIDENT_K,
  // not gate|up): every worker keeps its whole share in registers, requested before the wait, so
  // the stage's HBM traffic overlaps the stage before it and nothing has to be reduced over workers.
  {
    const int ux = (n_units + n_xcd - 1) / std::max(1, n_xcd), g = (ux + std::max(1, wpx) - 1) / std::max(1, wpx);
    if (!(flags & FLEET_FLAG_NO_RESIDENT) && nb == 1 && m_tiles == 1 && K <= RESIDENT_K && g <= RESIDENT_UNITS)
      return MfmaPlan{g, 1, 1};
  }
  if (msplit_applies(sched, P_MFMA, m_tiles, n_xcd)) {   // n_xcd / m_tiles XCDs share one m-tile and split N
    const int xpm = n_xcd / m_tiles;
    return plan_mfma((n_units + xpm - 1) / xpm, wpx, K, nb, mfma_blocks(tile_m), 1, split_ok);
  }
  return plan_mfma((n_units + n_xcd - 1) / std::max(1, n_xcd), wpx, K, nb, mfma_blocks(tile_m), m_tiles, split_ok);
}

// Largest batch that runs the FMA GEMV kernels.  Measured on MI355X the MFMA kernels (with the
// RMSNorm fused into them) win from batch 2 on (12 layers, per step: batch 1 0.984 ms FMA / 1.080
// ms MFMA, batch 2 1.147 / 1.104), so the default is 1; the environment variable
// FLEET_FMA_MAX_BATCH (0..8) moves the switch, e.g. to 8 for FMA at batch 2-8.
int fma_max_from_env() {
  const char* e = getenv("FLEET_FMA_MAX_BATCH");
  if (!e) return 1;
  return std::min(8, std::max(0, atoi(e)));
}

int resolve_tile_m(int batch, int tile_m, int fma_max) {
  if (batch <= fma_max) return batch;  // FMA GEMV path: one tile holds the whole batch
  if (tile_m == 0) return std::min(MAX_TILE_ROWS, ((batch + 15) / 16) * 16);
  return tile_m;
}

int attention_splits(int batch, int n_kv_heads, int n_workers, int max_seq) {
  // as many splits as there are idle workers, but no split shorter than about 100 cache slots
  // (measured at batch 1: a capacity of 1001 slots runs 2 % faster with 8 splits than with 4, 1025 slots 7 % slower with 16 than with 8)
  // (a split costs a fixed prologue and its partial has to be merged)
  int pairs = std::max(1, batch * n_kv_heads);
  int s = 1;
  while (s * 2 <= 32 && pairs * s * 2 <= n_workers && s * 2 * 100 <= max_seq) s *= 2;
  return s;
}

int check_shape(const fleet_shape_t& s) {
  if (s.n_layers < 1 || s.n_layers > MAX_LAYERS || s.hidden < 32 || s.ffn < 32 || s.n_q_heads < 1 || s.n_kv_heads < 1) return FLEET_EINVAL;
  if (s.head_dim != 128) return FLEET_EINVAL;
  if (s.n_q_heads % s.n_kv_heads || s.n_q_heads / s.n_kv_heads > 4) return FLEET_EINVAL;
  if (s.hidden % 32 || s.ffn % 32) return FLEET_EINVAL;
  if (s.vocab < 0 || s.vocab % 16) return FLEET_EINVAL;
  if (s.max_batch < 1 || s.max_batch > MAX_BATCH || s.max_seq < 1) return FLEET_EINVAL;
  // the kernels address one weight matrix, and one (sequence, kv head) stream of the cache,
  // with 32-bit byte offsets
  const int64_t lim = (int64_t)1 << 31;
  const int64_t H = s.hidden, F = s.ffn, QD = (int64_t)s.n_q_heads * s.head_dim;
  const int64_t NQKV = (int64_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
  if (NQKV * H * 2 >= lim || QD * H * 2 >= lim || 2 * F * H * 2 >= lim || (int64_t)s.vocab * H * 2 >= lim) return FLEET_EINVAL;
  if ((int64_t)s.max_seq * s.head_dim * 2 >= lim) return FLEET_EINVAL;
  // one arrival counter per (sequence, kv head) for the split-KV merge
  if ((int64_t)s.max_batch * s.n_kv_heads > MAX_BATCH * 8) return FLEET_EINVAL;
  if (s.sched_mode < FLEET_SCHED_COOPERATIVE || s.sched_mode > FLEET_SCHED_MSPLIT) return FLEET_EINVAL;
  if (s.tile_m != 0 && s.tile_m != 16 && s.tile_m != 32 && s.tile_m != 64) return FLEET_EINVAL;
  if (!(s.rms_eps >= 0.f) || !(s.rope_theta > 0.f)) return FLEET_EINVAL;
  return FLEET_OK;
}

Graph build_decode_graph(const fleet_shape_t& s, int batch, int n_xcd, int n_workers, bool loop, int fma_max) {
  Builder b(n_xcd, n_workers, s.sched_mode, batch);
  const int H = s.hidden, hd = s.head_dim, nq = s.n_q_heads, nkv = s.n_kv_heads, F = s.ffn;
  const int QD = nq * hd, NQKV = (nq + 2 * nkv) * hd;
  const Path path = batch <= fma_max ? P_FMA : P_MFMA;
  const int ur = path == P_FMA ? 8 : 16;
  const int tm = resolve_tile_m(batch, s.tile_m, fma_max);
  const int mt = (batch + tm - 1) / tm;
  const int S = attention_splits(batch, nkv, n_workers, s.max_seq);

  // MFMA operators carry their tile plan in aux2: bits 12..15 units per tile, 16..19 k-slices
  auto plan_bits = [&](int n_units, int K, int nb) {
    if (path != P_MFMA) return 0;
    const MfmaPlan pl = plan_for(s.sched_mode, s.flags, n_units, K, nb, tm, mt, n_xcd, n_workers);
    return (pl.G << 12) | (pl.KS << 16) | (pl.resident << 21);
  };

  auto row_key = [](int i) { return i; };
  auto row_arg = [](int i, int* a) { a[0] = i; a[1] = a[2] = a[3] = 0; };

  // stage: ingest (bf16 hidden or embedding gather -> fp32 residual stream)
  b.mark_all();
  int op_in = b.add_op(B_INGEST, -1, E_STORE_F32, P_FMA, H, H, 0, 0, 1, batch, BUF_HIDDEN_IN, BUF_X, 0, W_EMBED);
  int ev = b.cu_stage(op_in, batch, -1, row_key, row_arg);
  b.g.xready.push_back(ev);

  // FMA path: the RMSNorm is fused into the GEMV that consumes it (every worker
  // normalises the L2-resident residual rows into LDS); MFMA path: CU-task per row
  const bool fuse_norm = path == P_FMA && !(s.flags & FLEET_FLAG_SEPARATE_NORM) &&
                         (int64_t)batch * H * 2 <= GEMV_LDS_X_BYTES;
  // MFMA path, tiles of 16 batch rows: fused as well.  The GEMM reads the fp32 residual rows and
  // scales them into its bf16 operands itself; the sums of squares come from the epilogues that
  // wrote the rows (one partial per row and 16 features, BUF_SS).  Taller tiles have no
  // registers left for fp32 operands and keep the norm stages.
  const bool fuse_norm_mfma = path == P_MFMA && !(s.flags & FLEET_FLAG_SEPARATE_NORM) &&
                              mfma_blocks(tm) <= FUSED_NORM_MAX_BLOCKS && H % 64 == 0 && H <= 32768;
  auto xmode = [&](int K) { return path == P_FMA && (int64_t)batch * K * 2 <= GEMV_LDS_X_BYTES ? X_LDS_COPY : X_GLOBAL; };
  // weight blocks requested before the wait (bits 10..11 of aux2).  Measured at batch 1:
  // requesting only one block after the short O-projection stage (to reach the poll
  // sooner) is slower than requesting the full depth everywhere.
  const int PRE2 = 3 << 10;

  // FMA path: the workers that run an XCD's attention tasks (its first ranks: the tasks are
  // dealt by rank) take no units of the O projection when they are at most half of the XCD's
  // workers.  The others hold their O weights before attention ends, so the O stage does not
  // wait for the attention workers to fetch theirs.
  std::vector<int> o_skip(n_xcd, 0);
  if (s.sched_mode != FLEET_SCHED_UNAWARE)
    for (int x = 0; x < n_xcd; ++x) {
      int n_att = 0;
      for (int p = 0; p < batch * nkv; ++p) n_att += (p % n_xcd == x) ? S : 0;
      const int wpx = n_workers / std::max(1, n_xcd);
      o_skip[x] = 2 * n_att <= wpx ? n_att : 0;
    }

  for (int l = 0; l < s.n_layers; ++l) {
    b.mark_all();
    int op_qkv;
    if (fuse_norm) {
      op_qkv = b.add_op(B_GEMM, l, E_STORE_F32, path, H, NQKV, ur, NQKV / ur, mt, tm, BUF_X, BUF_QKV, 0, W_QKV,
                        W_LN1 | (X_LDS_NORM << 8) | PRE2);   // FMA path only
    } else if (fuse_norm_mfma) {
      op_qkv = b.add_op(B_GEMM, l, E_STORE_F32, path, H, NQKV, ur, NQKV / ur, mt, tm, BUF_X, BUF_QKV, 0, W_QKV,
                        W_LN1 | PRE2 | AUX2_FUSED_NORM | plan_bits(NQKV / ur, H, 1));
    } else {
      // the norm tasks go to the XCD's highest ranks: where the QKV weights stay in registers the
      // lowest ranks hold the tiles and request their whole share before the wait -- a worker
      // that ran a norm task first would request it late and end the QKV stage late
      int op_n1 = b.add_op(B_RMSNORM, l, E_STORE_F32, P_FMA, H, H, 0, 0, 1, batch, BUF_X, BUF_N, 0, W_LN1);
      // (up to four tasks per XCD; measured: batch 8 -3.6 %, batch 32 -0.5 %, batch 64 +1.2 % per step)
      ev = b.cu_stage(op_n1, batch, ev, row_key, row_arg, 1, batch <= 4 * n_xcd);
      op_qkv = b.add_op(B_GEMM, l, E_STORE_F32, path, H, NQKV, ur, NQKV / ur, mt, tm, BUF_N, BUF_QKV, 0, W_QKV,
                        (xmode(H) << 8) | PRE2 | plan_bits(NQKV / ur, H, 1));
    }
    // FMA path: where the attention workers are at most a quarter of every XCD's workers they
    // take no units of the QKV projection either: they have their first keys and values and
    // poll the QKV event when it fires, instead of coming to their attention task from the
    // tail of the stage it waits for (measured at batch 1: -0.55 % per step with 8 of 32
    // workers, +-0 with 16)
    bool qkv_skip = path == P_FMA && s.sched_mode != FLEET_SCHED_UNAWARE;
    for (int x = 0; x < n_xcd; ++x) qkv_skip = qkv_skip && o_skip[x] > 0 && 4 * o_skip[x] <= n_workers / std::max(1, n_xcd);
    ev = b.gemm_stage(op_qkv, ev, qkv_skip ? &o_skip : nullptr);

    // split-KV attention; the split that finishes last merges (no merge stage)
    int op_att = b.add_op(B_ATTN, l, E_STORE_F32, P_FMA, hd, QD, 0, 0, 1, batch, BUF_QKV, BUF_ATT, S, W_NONE);
    ev = b.cu_stage(op_att, batch * nkv * S, ev,
                    [S](int i) { return i / S; },
                    [S, nkv](int i, int* a) { int p = i / S; a[0] = p / nkv; a[1] = p % nkv; a[2] = i % S; a[3] = S; },
                    // every direct signal is 17 atomics (the device counter and its copies):
                    // measured, two-level pays for attention only with many tasks per XCD
                    ATTN_TWO_LEVEL_MIN_PER_XCD);

    // FMA path, cooperative: the O projection's idle workers warm the L2 with the first weight
    // block of their gate/up task while attention runs (aux = gate rows, low byte of aux2 =
    // W_GU: the op's second pointer is that matrix)
    // -- worth it only while most of the XCD idles through attention: attention workers at
    // most a quarter of each XCD's workers (batch 1 of the 8-KV-head model)
    bool warm_gu = path == P_FMA && s.sched_mode != FLEET_SCHED_UNAWARE;
    for (int x = 0; x < n_xcd; ++x) warm_gu = warm_gu && o_skip[x] > 0 && 4 * o_skip[x] <= n_workers / std::max(1, n_xcd);
    int op_o = b.add_op(B_GEMM, l, E_RESID_F32, path, QD, H, ur, H / ur, mt, tm, BUF_ATT, BUF_X, warm_gu ? F : 0, W_O,
                      (warm_gu ? W_GU : 0) | (xmode(QD) << 8) | PRE2 | plan_bits(H / ur, QD, 1));
    ev = b.gemm_stage(op_o, ev, path == P_FMA ? &o_skip : nullptr);

    // gate | up rows of one concatenated matrix; a unit is ur gate rows plus the
    // matching ur up rows (aux = row offset of the up half), SwiGLU in the epilogue
    // FLEET_FLAG_UNFUSED_SILU: a plain GEMM over all 2 * ffn rows stores fp32 sums, and a
    // stage of CU-tasks (one per sequence) applies SiLU(gate) x up afterwards.
    const bool unfused = (s.flags & FLEET_FLAG_UNFUSED_SILU) != 0;
    const Epi gu_epi = unfused ? E_STORE_F32 : E_SWIGLU_BF16;
    const int gu_n = unfused ? 2 * F : F, gu_aux = unfused ? 0 : F, gu_nb = unfused ? 1 : 2;
    const Buf gu_out = unfused ? BUF_GU32 : BUF_H;
    int op_gu;
    if (fuse_norm) {
      op_gu = b.add_op(B_GEMM, l, gu_epi, path, H, gu_n, ur, gu_n / ur, mt, tm, BUF_X, gu_out, gu_aux, W_GU,
                       W_LN2 | (X_LDS_NORM << 8) | PRE2);
    } else if (fuse_norm_mfma) {
      op_gu = b.add_op(B_GEMM, l, gu_epi, path, H, gu_n, ur, gu_n / ur, mt, tm, BUF_X, gu_out, gu_aux, W_GU,
                       W_LN2 | PRE2 | AUX2_FUSED_NORM | plan_bits(gu_n / ur, H, gu_nb));
    } else {
      int op_n2 = b.add_op(B_RMSNORM, l, E_STORE_F32, P_FMA, H, H, 0, 0, 1, batch, BUF_X, BUF_N, 0, W_LN2);
      ev = b.cu_stage(op_n2, batch, ev, row_key, row_arg);
      op_gu = b.add_op(B_GEMM, l, gu_epi, path, H, gu_n, ur, gu_n / ur, mt, tm, BUF_N, gu_out, gu_aux, W_GU,
                       (xmode(H) << 8) | PRE2 | plan_bits(gu_n / ur, H, gu_nb));
    }
    ev = b.gemm_stage(op_gu, ev);
    if (unfused) {
      int op_sw = b.add_op(B_SWIGLU, l, E_SWIGLU_BF16, P_FMA, F, F, 0, 0, 1, batch, BUF_GU32, BUF_H, F, W_NONE);
      ev = b.cu_stage(op_sw, batch, ev, row_key, row_arg);
    }

    int op_dn = b.add_op(B_GEMM, l, E_RESID_F32, path, F, H, ur, H / ur, mt, tm, BUF_H, BUF_X, 0, W_DOWN,
                      (xmode(F) << 8) | PRE2 | plan_bits(H / ur, F, 1));
    ev = b.gemm_stage(op_dn, ev);
    b.g.xready.push_back(ev);
  }

  // final stage: residual stream -> hidden_out, final norm -> BUF_N, then the LM head
  b.mark_all();
  int op_fin = b.add_op(B_FINAL, -1, E_STORE_F32, P_FMA, H, H, 0, 0, 1, batch, BUF_X, BUF_N,
                        s.vocab > 0 ? 1 : 0, W_FINAL);
  ev = b.cu_stage(op_fin, batch, ev, row_key, row_arg);
  b.mark_all();   // a step without logits ends here
  if (s.vocab > 0) {
    int op_lm = b.add_op(B_GEMM, -1, E_STORE_F32, path, H, s.vocab, ur, s.vocab / ur, mt, tm, BUF_N,
                         BUF_LOGITS, 0, W_LM, (xmode(H) << 8) | PRE2 | plan_bits(s.vocab / ur, H, 1));
    ev = b.gemm_stage(op_lm, ev);
    if (loop) {   // greedy next token per sequence; its event is the graph's last
      int op_am = b.add_op(B_ARGMAX, -1, E_STORE_F32, P_FMA, s.vocab, s.vocab, 0, 0, 1, batch, BUF_LOGITS, BUF_TOKENS, 0, W_NONE);
      ev = b.cu_stage(op_am, batch, ev, row_key, row_arg);
    }
  }
  b.mark_all();
  return b.finish(s.n_layers, tm, path, S, mt);
}

Graph build_gemm_graph(int B, int K, int N, int sched_mode, int tile_m, int flags, int reps,
                       int n_copies, int n_xcd, int n_workers, int fma_max) {
  Builder b(n_xcd, n_workers, sched_mode, B);
  const Path path = B <= fma_max ? P_FMA : P_MFMA;
  const int ur = path == P_FMA ? 8 : 16;
  const int tm = resolve_tile_m(B, tile_m, fma_max);
  const int mt = (B + tm - 1) / tm;
  int ev = -1;
  b.mark_all();
  b.mark_all();
  // Repetitions are independent unless FLEET_FLAG_CHAINED is set.  Split-K tiles count
  // their arrivals in one of two counter sets (bit 20 of aux2), so a repetition of such a
  // plan waits for the one before the previous: at most two are in flight.
  MfmaPlan pl{1, 1, 0};
  if (path == P_MFMA) pl = plan_for(sched_mode, flags, N / ur, K, 1, tm, mt, n_xcd, n_workers);
  std::vector<int> evs;
  for (int r = 0; r < reps; ++r) {
    const int xm = path == P_FMA && (int64_t)B * K * 2 <= GEMV_LDS_X_BYTES && !(flags & FLEET_FLAG_SEPARATE_NORM)
                       ? X_LDS_COPY : X_GLOBAL;
    const int bits = path == P_MFMA ? (pl.G << 12) | (pl.KS << 16) | ((r & 1) << 20) | (pl.resident << 21) : 0;
    int op = b.add_op(B_GEMM, r % std::max(1, n_copies), E_STORE_F32, path, K, N, ur, N / ur, mt, tm,
                      BUF_GEMM_X, BUF_GEMM_Y, 0, W_GEMM_COPY, (xm << 8) | (3 << 10) | bits);
    int wait = (flags & FLEET_FLAG_CHAINED) ? ev : (pl.KS > 1 && r >= 2) ? evs[r - 2] : -1;
    ev = b.gemm_stage(op, wait);
    evs.push_back(ev);
  }
  b.mark_all();
  b.mark_all();
  b.g.xready.push_back(-1);
  return b.finish(0, tm, path, 1, mt);
}

}  // namespace fleetg
