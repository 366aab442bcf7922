// Host-side task-graph builder for the decode-step megakernel.
//
// The graph follows the task model of paper section 3.1: every operator of a
// layer (section 2.2) becomes one device-task, made of chiplet-tasks (GEMMs in
// the cooperative schedule, one per XCD, section 3.2) or of CU-tasks (norms,
// attention, and every GEMM tile of the chiplet-unaware schedule).  Tasks name
// the event they wait for and the event they signal.  Everything is plain
// int32 words so that the graph can be dumped, compared and uploaded as is.
//
// Serialized layout (int32 words, in this order):
//   header [HEADER_WORDS]
//   ops    [n_ops   ][OP_WORDS]
//   tasks  [n_tasks ][TASK_WORDS]
//   events [n_events][EVENT_WORDS]
//   qoff   [n_xcd + 1]                  first queue entry of each XCD's queue
//   qents  [n_qent  ][QENT_WORDS]       the per-XCD queues, concatenated
//   marks  [n_xcd][n_layers + 4]        queue index (within the XCD's queue) of:
//                                       ingest, layer 0..L-1, final stage, LM head, end
//   xready [n_layers + 1]               event after which the residual stream
//                                       entering layer l is complete
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/fleet.h"

namespace fleetg {

constexpr int HEADER_WORDS = 32, OP_WORDS = 16, TASK_WORDS = 16, EVENT_WORDS = 4, QENT_WORDS = 4;
constexpr int32_t MAGIC = 0x464c5447;  // "FLTG"

// header word indices
enum {
  H_MAGIC = 0, H_VERSION, H_N_OPS, H_N_TASKS, H_N_EVENTS, H_N_XCD, H_N_QENT, H_N_LAYERS,
  H_BATCH, H_SCHED, H_TILE_M, H_PATH, H_N_SPLITS, H_N_WORKERS, H_M_TILES, H_TOTAL_WORDS
};

enum Body { B_INGEST = 0, B_RMSNORM = 1, B_GEMM = 2, B_ATTN = 3, B_SWIGLU = 4, B_FINAL = 5, B_ARGMAX = 6 };
enum Epi { E_STORE_F32 = 0, E_RESID_F32 = 1, E_SWIGLU_BF16 = 2 };
enum Path { P_FMA = 0, P_MFMA = 1 };
enum Scope { S_WAVE = 0, S_CU = 1, S_CHIPLET = 2 };
// how a queue entry's tasks reach the workers: every worker of the XCD runs the (one) task;
// dealt round-robin over the XCD's workers from rank 0 up, or (D_XCD_RR_TOP) from the highest
// rank down; dealt over all workers of the device
enum Dist { D_CHIPLET = 0, D_XCD_RR = 1, D_DEV_RR = 2, D_XCD_RR_TOP = 3 };
// EV_TWO_LEVEL: signalled by the workers of chiplet-tasks; EV_TWO_LEVEL_CU: by CU-tasks
// grouped per XCD (cooperative schedule); EV_DIRECT: by CU-tasks running anywhere
enum EventKind { EV_DIRECT = 0, EV_TWO_LEVEL = 1, EV_TWO_LEVEL_CU = 2 };
// a stage of CU-tasks signals two-level when it has more than one task per XCD on average
// (attention stages: more than this many -- measured: with up to 32 tasks per XCD the direct
// signals are 1 % of a step faster at batch 2 and 8, the same at batch 32)
constexpr int ATTN_TWO_LEVEL_MIN_PER_XCD = 32;

// activation / caller buffers, resolved to pointers per step
enum Buf {
  BUF_NONE = 0, BUF_X, BUF_N, BUF_QKV, BUF_ATT, BUF_H, BUF_PART, BUF_HIDDEN_IN, BUF_TOKENS,
  BUF_KC, BUF_VC, BUF_POS, BUF_HIDDEN_OUT, BUF_LOGITS, BUF_GEMM_X, BUF_GEMM_Y, BUF_GPART, BUF_GU32, BUF_TOKENS_OUT, BUF_PT,
  BUF_SS,   // fp32 [batch][hidden / 16]: sums of squares of the residual stream, one per row and 16 features
  N_BUF
};

// which caller weight an op reads (resolved with the op's layer)
enum WKind {
  W_NONE = 0, W_QKV, W_O, W_GU, W_DOWN, W_LM, W_LN1, W_LN2, W_FINAL, W_EMBED, W_GEMM_COPY
};

// op word indices
enum {
  O_BODY = 0, O_LAYER, O_EPI, O_PATH, O_K, O_N, O_UNIT_ROWS, O_N_UNITS, O_M_TILES, O_TILE_M,
  O_IN_BUF, O_OUT_BUF, O_AUX, O_WKIND, O_BATCH, O_AUX2
};
// O_AUX2 of a GEMM op: low byte = WKind of the op's second pointer (W_NONE if none): the gain
// of the fused RMSNorm (activation mode X_LDS_NORM), else the weights of the next GEMM, whose
// first block the op's idle workers pull into the L2 (O_AUX then holds that matrix's gate rows),
// bits 8..9 = activation mode of the FMA path (XMode), bits 10..11 = weight blocks the FMA
// path requests before its dependency wait (0..3); MFMA path: bits 12..15 = units per tile,
// bits 16..19 = k-slices of the split-K plan (1 = no split), bit 20 = counter set of the
// split-K arrival counters (isolated GEMM repetitions alternate), bit 21 = register-resident
// weights (MfmaPlan::resident), bit 22 = the op reads the fp32 residual stream and normalises
// it itself (RMSNorm fused into the MFMA GEMM; the gain is the op's second pointer)
constexpr int AUX2_FUSED_NORM = 1 << 22;
constexpr int FUSED_NORM_MAX_BLOCKS = 1;   // tallest tile (in blocks of 16 batch rows) whose kernel flavour has the fused norm
enum XMode { X_GLOBAL = 0, X_LDS_COPY = 1, X_LDS_NORM = 2 };
constexpr int GEMV_LDS_X_BYTES = 96 * 1024;   // LDS the FMA path may fill with activations
// task word indices.  A0..A3 by body:
//   GEMM chiplet-task : A0 first unit, A1 unit count, A2 workers (lowest ranks) that take
//                       no units (FMA path), A3 = m-tile + 1 if the task covers one m-tile
//                       only (M-split), else 0                 (tiles = units x m_tiles)
//   GEMM CU-task      : A0 first unit, A1 unit count, A2 m-tile, A3 k-slice
//   ATTN              : A0 batch row, A1 kv head, A2 split, A3 n_splits
//   INGEST/RMSNORM/SWIGLU/FINAL/ARGMAX : A0 batch row
enum { T_OP = 0, T_SCOPE, T_XCD, T_A0, T_A1, T_A2, T_A3, T_WAIT_EVENT, T_SIGNAL_EVENT, T_STAGE };
// event word indices: threshold counts device-level signals (XCDs for a
// two-level event, tasks for a direct one); n_tasks counts the signalling tasks
enum { E_THRESHOLD = 0, E_KIND, E_XCD_MASK, E_N_TASKS };
// queue entry word indices
enum { Q_FIRST = 0, Q_COUNT, Q_DIST, Q_STAGE };

struct Graph {
  std::vector<int32_t> header, ops, tasks, events, qoff, qents, marks, xready;
  int n_ops() const { return (int)ops.size() / OP_WORDS; }
  int n_tasks() const { return (int)tasks.size() / TASK_WORDS; }
  int n_events() const { return (int)events.size() / EVENT_WORDS; }
  int n_qent() const { return (int)qents.size() / QENT_WORDS; }
  std::vector<int32_t> serialize() const;
};

// Tile plan of an MFMA GEMM operator (units per tile, k-slices); a split-K plan needs one
// arrival counter per (first unit of a tile, m-tile), GEMM_TILE_COUNTERS at most
constexpr int GEMM_TILE_COUNTERS = 4096;
// resident = 1: the operator's weight share per worker (at most RESIDENT_UNITS units, K up to
// RESIDENT_K) is held in registers whole, requested before the dependency wait; one k-slice
constexpr int RESIDENT_UNITS = 2, RESIDENT_K = 4096;
struct MfmaPlan { int G, KS, resident; };
MfmaPlan plan_mfma(int units_per_xcd, int workers_per_xcd, int K, int nb, int mt_blocks, int m_tiles, bool allow_split);
// 16-row blocks of batch rows the MFMA kernel for tile height tile_m accumulates (1, 2 or 4)
int mfma_blocks(int tile_m);
// largest batch that runs the FMA GEMV kernels (larger batches run the MFMA kernels): 1, or
// what the environment variable FLEET_FMA_MAX_BATCH (0..8) says.  Read once by whoever owns
// a set of graphs (fleet_create, fleet_gemm, fleet_graph_build) and handed to the builders, so
// that the graphs and the packed weight copies of one owner always agree.
int fma_max_from_env();
constexpr int MAX_TILE_ROWS = 64;   // batch rows one MFMA tile can hold (4 blocks of 16)
constexpr int MAX_BATCH = 128;
constexpr int MAX_LAYERS = 120;     // at most 8 events per layer: a graph stays within the 1024 entries of the kernels' event table
// tile_m actually used for `batch` (0 = whole batch rounded up to 16, at most MAX_TILE_ROWS;
// FMA path: batch)
int resolve_tile_m(int batch, int tile_m, int fma_max);
// KV splits per (sequence, kv head)
int attention_splits(int batch, int n_kv_heads, int n_workers, int max_seq);
// validate a shape; returns FLEET_OK or FLEET_EINVAL
int check_shape(const fleet_shape_t& s);

// the decode-step graph for `batch` sequences on n_xcd chiplets, n_workers workgroups
// loop = true: a last stage of ARGMAX CU-tasks (greedy next token, one per sequence) so that a
// launch can run several decode steps back to back
Graph build_decode_graph(const fleet_shape_t& s, int batch, int n_xcd, int n_workers, bool loop, int fma_max);
// `reps` GEMM device-tasks y = x W^T (rep i reads weight copy i % n_copies)
Graph build_gemm_graph(int B, int K, int N, int sched_mode, int tile_m, int flags, int reps,
                       int n_copies, int n_xcd, int n_workers, int fma_max);
// marks per XCD of a decode graph with n_layers layers
inline int n_marks(int n_layers) { return n_layers + 4; }

}  // namespace fleetg
