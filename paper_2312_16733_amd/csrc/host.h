// Host-side state of a resident SuperNet and of one forward call.
#pragma once
#include <array>
#include <map>
#include <string>
#include <vector>

#include "common.h"

namespace sna {

constexpr int NBUF = 8;              // activation buffers per group in the arena
constexpr float SN_EPS = 1e-5f;

struct ArchTables {
  sna_arch_desc arch;
  std::vector<sna_tensor_info> tensors;
  std::vector<sna_norm_info> norms;
  std::map<std::string, int> tidx, nidx;
  int64_t weight_bytes = 0;
  int64_t row_len = 0;
  int64_t per_image_elems = 0;       // largest activation of one request, in elements
  int64_t in_elems_max = 0;          // largest request input, in elements
  int64_t small_elems = 0;           // per-request fp32 scratch (pooled vectors, gates, logits)
  int esz = 2;                       // bytes per stored activation / weight element
};

sna_status build_tables(const sna_arch_desc* arch, ArchTables* t);
sna_status fail(sna_status st, const char* fmt, ...);

// Tuning table key: (M, K_out, C_in, taps, stride, parts, same-shaped problems sharing the launch)
typedef std::array<int, 7> TuneKey;

struct ProfRec {
  int kc; hipEvent_t a, b; std::string what;
  double flops = 0, bytes = 0;       // algorithmic work of the launch
  bool igemm = false;                // a matrix-kernel launch: `key` is the tuning key of its problem with the most work
  int variant = -1;                  // the tile variant that launch ran with
  TuneKey key{};
};

struct Group {
  const sna_subnet_cfg* cfg = nullptr;
  int cfg_index = 0;
  int n = 0;                         // requests routed to this cfg
  std::vector<int> reqs;             // their positions in the call, ascending
  bool contiguous = true;
  bool raw_input = false;            // cur points at the caller's unpadded request images
  char* buf[NBUF] = {nullptr};
  char* inbuf = nullptr;
  float* small = nullptr;
  // running state of the activation handed from layer to layer
  const void* cur = nullptr;
  int H = 0, W = 0, C = 0;
  int cur_buf = -1;
};

// One recorded kernel launch of a forward call.
struct PlanOp {
  enum Type { IGEMM, KREDUCE, DIRECT, MAXPOOL, GAP, DW, SE, LN, ATTN, COPY, PAD, STEMPOOL, MBV3HEAD, NORMCAL, NORMAPPLY } type;
  int variant = 0, flag = 0;         // igemm: tile variant, chunked kernel; direct / pool: dtype
  int kc = 0;                        // kernel class for the per-launch timing
  double flops = 0, bytes = 0;
  std::vector<char> args;            // the launcher's argument struct
};
// A pointer field inside an op's arguments that points into a caller buffer of the forward call
// (inputs, logits, hidden) rather than into the resident workspace: rewritten on every replay.
struct PlanPatch { int op; int offset; int which; size_t delta; };
struct Plan {
  std::string key;                   // everything the launch list depends on, byte for byte
  std::vector<PlanOp> ops;
  std::vector<PlanPatch> patches;
  int64_t macs = 0;
  uint64_t last_use = 0;
};

}  // namespace sna

struct sna_supernet {
  sna::ArchTables T;
  const char* weights = nullptr;
  const float* stats = nullptr;
  char* workspace = nullptr;
  size_t workspace_bytes = 0;
  float* folded = nullptr;           // [n_subnets][2][row_len]
  char* arena = nullptr;
  size_t arena_bytes = 0;
  char* partials = nullptr;          // fp32 K-chunk sums of split reductions (raw layer outputs while calibrating)
  size_t partials_bytes = 0;
  int* counters = nullptr;           // kTileCounters ints, all zero between launches (in-kernel split reductions)
  int split_mode = 0;                // 0 auto, 1 never split a reduction over blocks, 2 always when chunked
  // tile variant measured best for a layer shape: (M, K_out, C_in, R*S, stride, parts) -> variant
  std::map<sna::TuneKey, int> tuned;
  // measured for a chunked layer shape: 1 = one block per K chunk plus the reduction kernel is faster
  std::map<sna::TuneKey, int> tuned_split;
  // SubnetNorm calibration in progress: every layer with statistics keeps its raw output, measures it
  // and writes the subnet's row of the caller's table (stats_mut) before normalising
  bool calibrating = false;
  float* stats_mut = nullptr;
  int forced_variant = -1;           // >= 0: every igemm launch uses this tile variant (test knob)
  bool tuning = false;               // the forward in progress measures shapes it has no entry for
  // launch lists of recent forward calls, replayed when the same cfgs / routing come again
  std::vector<sna::Plan> plans;
  uint64_t plan_clock = 0;
  bool plan_cache_on = true;
  int n_subnets = 0, max_batch = 0;
  // bookkeeping of the last forward
  int64_t last_macs = 0;
  int last_launches = 0;
  // per-launch event timing
  bool prof_on = false;
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  std::vector<sna::ProfRec> prof_recs;
  double prof_flops[SNA_N_KCLASS] = {0}, prof_bytes[SNA_N_KCLASS] = {0};
  int64_t prof_launches[SNA_N_KCLASS] = {0};
};
