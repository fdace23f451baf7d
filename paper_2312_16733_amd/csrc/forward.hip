// C ABI and the host-side planner: validates the control tuples, groups requests by cfg, walks
// the SuperNet in layer order and issues one grouped launch per layer slot.  LayerSelect is
// decided here: a block beyond a cfg's depth produces no problem, hence no launch and no copy.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <set>

#include "host.h"

namespace sna {
const char* last_error_text();

static inline int out_size(int h, int k, int stride) { return (h + 2 * (k / 2) - k) / stride + 1; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------
// cfg validation
// ------------------------------------------------------------------------------------------
static sna_status check_ch(int v, int mx, const char* what, int s, int j) {
  if (v < 8 || v > mx) return fail(SNA_E_CFG_RANGE, "%s[%d][%d]=%d outside [8, %d]", what, s, j, v, mx);
  if (v % 8) return fail(SNA_E_CFG_ALIGN, "%s[%d][%d]=%d is not a multiple of 8", what, s, j, v);
  return SNA_OK;
}

static sna_status validate_cfg(const sna_supernet* net, const sna_subnet_cfg& c) {
  const sna_arch_desc& a = net->T.arch;
  if (c.subnet_id < 0 || c.subnet_id >= net->n_subnets)
    return fail(SNA_E_SUBNET_ID, "subnet_id %d outside [0, %d)", c.subnet_id, net->n_subnets);
  sna_status st;
  if (a.family == SNA_FAMILY_TRANSFORMER) {
    if (c.n_stages != 1) return fail(SNA_E_CFG_RANGE, "n_stages %d != 1", c.n_stages);
    if (c.depth[0] < 1 || c.depth[0] > a.max_layers) return fail(SNA_E_CFG_RANGE, "depth %d", c.depth[0]);
    if (c.in_h != a.seq_len) return fail(SNA_E_CFG_RANGE, "tokens %d != seq_len %d", c.in_h, a.seq_len);
    for (int j = 0; j < c.depth[0]; ++j) {
      const int at = c.block_mid_ch[0][j], ff = c.block_aux_ch[0][j];
      if (at < a.head_dim || at > a.n_heads * a.head_dim || at % a.head_dim)
        return fail(SNA_E_CFG_RANGE, "layer %d attention width %d", j, at);
      if ((st = check_ch(ff, a.ffn, "ffn", 0, j)) != SNA_OK) return st;
    }
    return SNA_OK;
  }
  if (c.n_stages != a.n_stages) return fail(SNA_E_CFG_RANGE, "n_stages %d != %d", c.n_stages, a.n_stages);
  if (c.in_h < 8 || c.in_h > a.max_res || c.in_w < 8 || c.in_w > a.max_res)
    return fail(SNA_E_CFG_RANGE, "resolution %dx%d outside [8, %d]", c.in_h, c.in_w, a.max_res);
  if ((st = check_ch(c.stage_out_ch[0], a.stem_ch, "stem", 0, 0)) != SNA_OK) return st;
  if (a.family == SNA_FAMILY_MBV3 && c.stage_out_ch[0] != a.stem_ch)
    return fail(SNA_E_CFG_RANGE, "MBV3 stem width is fixed at %d", a.stem_ch);
  if (a.family == SNA_FAMILY_TINY && c.stage_out_ch[0] != a.stem_ch)
    return fail(SNA_E_CFG_RANGE, "TINY stem width is fixed at %d", a.stem_ch);
  for (int s = 0; s < a.n_stages; ++s) {
    if (c.depth[s] < 1 || c.depth[s] > a.stage_max_depth[s])
      return fail(SNA_E_CFG_RANGE, "depth[%d]=%d outside [1, %d]", s, c.depth[s], a.stage_max_depth[s]);
    if ((st = check_ch(c.stage_out_ch[1 + s], a.stage_ch[s], "stage_out_ch", s, 0)) != SNA_OK) return st;
    if (a.family == SNA_FAMILY_MBV3 && c.stage_out_ch[1 + s] != a.stage_ch[s])
      return fail(SNA_E_CFG_RANGE, "MBV3 stage widths are fixed");
    if (a.family == SNA_FAMILY_TINY) continue;
    for (int j = 0; j < c.depth[s]; ++j) {
      if ((st = check_ch(c.block_mid_ch[s][j], a.block_max_mid[s][j], "block_mid_ch", s, j)) != SNA_OK) return st;
      if (a.family == SNA_FAMILY_MBV3) {
        const int k = c.block_kernel[s][j];
        if (k != 3 && k != 5 && k != 7) return fail(SNA_E_CFG_RANGE, "block_kernel[%d][%d]=%d", s, j, k);
        if (a.stage_se[s] &&
            (st = check_ch(c.block_aux_ch[s][j], a.block_max_aux[s][j], "block_aux_ch", s, j)) != SNA_OK)
          return st;
      }
    }
  }
  return SNA_OK;
}

// ------------------------------------------------------------------------------------------
// one forward call
// ------------------------------------------------------------------------------------------
struct Fwd {
  sna_supernet* net;
  hipStream_t stream;
  std::vector<Group> groups;
  hipError_t err = hipSuccess;
  int64_t macs = 0;
  std::vector<PlanOp> ops;

  const ArchTables& T() const { return net->T; }
  int esz() const { return net->T.esz; }

  const sna_tensor_info& tensor(const std::string& name) const { return T().tensors[T().tidx.at(name)]; }
  const char* wptr(const sna_tensor_info& ti) const { return net->weights + ti.offset; }
  const float* scale_of(const std::string& norm, int subnet) const {
    const sna_norm_info& ni = T().norms[T().nidx.at(norm)];
    return net->folded + (size_t)subnet * 2 * T().row_len + ni.offset;
  }
  const float* shift_of(const std::string& norm, int subnet) const { return scale_of(norm, subnet) + T().row_len; }

  // ---- profiling brackets ------------------------------------------------------------------
  hipEvent_t next_event() {
    if (net->ev_used == net->ev_pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      net->ev_pool.push_back(e);
    }
    return net->ev_pool[net->ev_used++];
  }
  // Record one launch.  Nothing runs here: the list is executed (and kept for replay) afterwards.
  template <class A>
  void emit(PlanOp::Type type, int variant, int flag, int kc, double flops, double bytes, const A& a) {
    if (err != hipSuccess) return;
    ops.emplace_back();
    PlanOp& op = ops.back();
    op.type = type; op.variant = variant; op.flag = flag; op.kc = kc; op.flops = flops; op.bytes = bytes;
    op.args.resize(sizeof(A));
    memcpy(op.args.data(), &a, sizeof(A));
  }

  // ---- conv / linear ---------------------------------------------------------------------------
  // Fill the WeightSlice part of a problem: leading K x C block, centre ksize window of the
  // stored kernel, read at the stored tensor's strides.
  void slice_conv(ConvProblem& p, const sna_tensor_info& ti, int K, int ksize, int stride) {
    const int rmax = ti.kind == 0 ? ti.dims[1] : 1, smax = ti.kind == 0 ? ti.dims[2] : 1;
    const int cmax = ti.c_pad;
    p.wk = rmax * smax * cmax; p.wr = smax * cmax; p.ws = cmax;
    const int r0 = (rmax - ksize) / 2, s0 = (smax - ksize) / 2;
    p.w = wptr(ti) + ((size_t)r0 * p.wr + (size_t)s0 * p.ws) * (ti.dtype == SNA_DTYPE_BF16 ? 2 : 4);
    p.K = K; p.R = ksize; p.S = ksize; p.stride = stride; p.pad = ksize / 2;
    p.Ho = out_size(p.H, ksize, stride); p.Wo = out_size(p.W, ksize, stride);
    p.M = p.N * p.Ho * p.Wo;
    p.C8 = p.C / 8; p.K8 = p.R * p.S * p.C8;
    p.magic_wo = p.Wo > 1 ? (unsigned)((1ull << 32) / (unsigned)p.Wo + 1) : 0;
    p.magic_ho = p.Ho > 1 ? (unsigned)((1ull << 32) / (unsigned)p.Ho + 1) : 0;
    if ((double)p.M * (p.Wo > p.Ho ? p.Wo : p.Ho) >= 4294967296.0) err = hipErrorInvalidValue;   // reciprocal range
    p.inv_s = (65536 + p.S - 1) / p.S;
    p.parts = 1; p.tiles_base = 0; p.kt_part = 1 << 30; p.kt_chunk = 1 << 30; p.part_stride = 0;
    p.y_stride = K; p.res_stride = K;
    const int esize = ti.dtype == SNA_DTYPE_BF16 ? 2 : 4;
    const double xb = (double)p.N * p.H * p.W * p.C * esize, wb = (double)K * p.wk * esize;
    if (xb >= 2147483648.0 || wb >= 2147483648.0) err = hipErrorInvalidValue;   // 32-bit buffer offsets
    p.x_bytes = (unsigned)xb;
    p.w_bytes = (unsigned)(wb - ((size_t)r0 * p.wr + (size_t)s0 * p.ws) * esize);
  }

  // Tile choice (measured on MI355X): 128-row tiles with two blocks per CU; the column tile that
  // pads the active out-channels least, wider for deep reductions; 64-row tiles when a layer has
  // too few 128-row tiles to fill 256 CUs; 32 rows for head-sized M.
  static int pick_variant(int M, int K, int depth) {
    // variants: 0 128x128, 1 128x64, 2 128x96, 3 128x32, 4 64x64, 5 64x128, 6 32x128
    if (M <= 32) return 6;
    if (K <= 32) return 3;
    int bn = 128, best = 1 << 30;
    const int cand[3] = {128, 96, 64};
    for (int c : cand) {
      const int padded = (K + c - 1) / c * c;
      const bool better = padded < best || (padded == best && depth < 1024);   // ties: narrower for shallow K
      if (better) { best = padded; bn = c; }
    }
    const long tiles128 = (long)((M + 127) / 128) * ((K + bn - 1) / bn);
    if (tiles128 < 256) return K <= 64 ? 4 : 5;
    return bn == 128 ? 0 : (bn == 64 ? 1 : 2);
  }

  // Fill the launch-side fields of a problem for tile variant v (parts already decided).
  static void place(ConvProblem& q, int v) {
    int bm, bn;
    igemm_tile_shape(v, &bm, &bn);
    q.tiles_n = (q.K + bn - 1) / bn;
    q.tiles_base = ((q.M + bm - 1) / bm) * q.tiles_n;
    q.tiles = q.tiles_base * q.parts;
    // reduction inside the matrix kernel: the chunk sums are kept tile by tile (bm x bn floats each)
    if (q.counters) q.part_stride = (unsigned long)q.tiles_base * bm * bn * 4;
  }

  // Time every tile variant on this one problem (followed by its reduction launch when the
  // reduction is split over blocks) and return the fastest; *best_ms gets its time per run.
  // Runs the problem for real (outputs are rewritten with the same values each time) and
  // synchronises on the stream.
  int measure_variants(const ConvProblem& q, bool chunked, const ConvProblem* reduce, float* best_ms, int copies = 1) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { err = hipErrorUnknown; return 0; }
    ConvGroupArgs ra;
    if (reduce) {
      ra.n = 1;
      ra.p[0] = *reduce;
      ra.p[0].tiles = (int)(((long)reduce->M * (reduce->K / 8) + 255) / 256);
      ra.p[0].tile_start = 0;
      ra.total_tiles = ra.p[0].tiles;
    }
    int best = -1;
    *best_ms = 0.f;
    for (int v = 0; v < igemm_num_variants() && err == hipSuccess; ++v) {
      if (!igemm_variant_ok(v, q)) continue;
      ConvGroupArgs a;
      a.n = copies < 1 ? 1 : (copies > SNA_MAX_GROUPS ? SNA_MAX_GROUPS : copies);   // twins: the launch carries that many tiles
      a.total_tiles = 0;
      for (int c = 0; c < a.n; ++c) {
        a.p[c] = q;
        place(a.p[c], v);
        a.p[c].tile_start = a.total_tiles;
        a.total_tiles += a.p[c].tiles;
      }
      auto once = [&] {
        err = launch_igemm(a, v, chunked, stream);
        if (err == hipSuccess && reduce) err = launch_splitk_reduce(ra, stream);
      };
      once();                                            // loads the code object, warms the caches
      float v_ms = 0.f;
      for (int trial = 0; trial < 2 && err == hipSuccess; ++trial) {
        const int reps = 4;
        err = hipEventRecord(e0, stream);
        for (int r = 0; r < reps && err == hipSuccess; ++r) once();
        if (err == hipSuccess) err = hipEventRecord(e1, stream);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        ms /= reps;
        if (trial == 0 || ms < v_ms) v_ms = ms;
      }
      if (err == hipSuccess && (best < 0 || v_ms < *best_ms)) { best = v; *best_ms = v_ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return best < 0 ? 0 : best;
  }

  // `twins`: how many problems of this very shape share the launch (the Q, K and V projections of a layer):
  // a launch with three times the tiles wants another tile than the same shape launched alone
  static TuneKey tune_key(const ConvProblem& q, int parts, int twins) {
    return {q.M, q.K, q.C, q.R * q.S, q.stride, parts, twins};
  }

  // K chunking, a function of the reduction length only: the same layer of the same subnet is
  // summed in the same order whatever it is batched with and however its blocks are laid out.
  static int chunk_steps(int kt_all) {
    const int n = kt_all <= 24 ? 1 : (kt_all <= 64 ? 2 : 4);
    return (kt_all + n - 1) / n;
  }

  void run_igemm(std::vector<ConvProblem>& ps, bool unify = false) {
    if (ps.empty()) return;
    const size_t n = ps.size();
    std::vector<int> var(n), chunks(n), twins(n, 1);
    for (size_t i = 0; i < n; ++i) {
      int t = 0;
      for (size_t j = 0; j < n; ++j)
        t += ps[j].M == ps[i].M && ps[j].K == ps[i].K && ps[j].C == ps[i].C && ps[j].R == ps[i].R && ps[j].S == ps[i].S &&
             ps[j].stride == ps[i].stride;
      twins[i] = t;
    }
    // the table's entry for this shape with as many twins, else with the nearest smaller count (a mixed batch can
    // bring more same-shaped problems together than any single-subnet call that was measured)
    auto find_tuned = [&](const ConvProblem& q, int parts, int tw) {
      for (; tw >= 1; --tw) {
        auto it = net->tuned.find(tune_key(q, parts, tw));
        if (it != net->tuned.end()) return it;
      }
      return net->tuned.end();
    };
    long tiles_all = 0;
    for (size_t i = 0; i < n; ++i) {
      ConvProblem& q = ps[i];
      if (q.C % 8 || q.K % 8 || q.y_stride % 8 || q.res_stride % 8 || q.R * q.S > 64 ||
          (q.out_fp32 && (q.act != SNA_ACT_NONE || q.res))) {
        err = hipErrorInvalidValue;      // shapes the MFMA path does not take; callers route these elsewhere
        return;
      }
      q.parts = 1;
      q.kt_part = 1 << 30;
      auto it = find_tuned(q, 1, twins[i]);
      var[i] = it != net->tuned.end() ? it->second : pick_variant(q.M, q.K, q.C * q.R * q.S);
      place(q, var[i]);
      tiles_all += q.tiles_base;
      const int kt_all = (q.K8 + 7) / 8;
      q.kt_chunk = chunk_steps(kt_all);
      chunks[i] = (kt_all + q.kt_chunk - 1) / q.kt_chunk;
    }
    // Too few tiles for the chip: give every chunk its own blocks and sum them in a second launch
    // (a measured per-shape decision, where there is one, takes precedence).
    const bool split_rule = net->split_mode >= 2 || (net->split_mode == 0 && tiles_all < 256);
    std::vector<ConvProblem> reduce;
    char* part_cur = net->partials;
    size_t counters_used = 0;
    for (size_t i = 0; i < n; ++i) {
      ConvProblem& q = ps[i];
      // room for the chunk sums: row-major [chunks][M][K] for the separate reduction kernel; the matrix
      // kernel's own reduction keeps them tile by tile, rows and columns padded to the tile (at most
      // 128 x 192), so the larger of the two is reserved
      const size_t part_bytes = align_up((size_t)chunks[i] * (q.M + 128) * (q.K + 192) * 4, 256);
      const bool can_split = chunks[i] > 1 && (size_t)(part_cur - net->partials) + part_bytes <= net->partials_bytes;
      ConvProblem r = q, qs = q;         // the reduction finishes the layer: keeps y, norm, residual, activation
      if (can_split) {
        r.x = part_cur;
        r.parts = chunks[i];
        r.part_stride = (unsigned long)q.M * q.K * 4;
        qs.parts = chunks[i];
        qs.kt_part = q.kt_chunk;
        qs.part_stride = r.part_stride;
        qs.y = part_cur; qs.y_stride = q.K; qs.out_fp32 = 1;
        qs.scale = nullptr; qs.shift = nullptr; qs.res = nullptr; qs.act = SNA_ACT_NONE;
      }
      bool split = can_split && split_rule;
      // the reduction can finish inside the matrix launch when the layer's tile counters fit the table
      // (mode 3 keeps the separate reduction kernel: a test knob for that path)
      // (room is reserved for the smallest tile any variant has, 32 x 32; the slots are handed out below,
      // once the tile variant is final)
      const size_t counters_need = (size_t)((q.M + 31) / 32) * ((q.K + 31) / 32);
      const bool fuse_reduce = can_split && net->split_mode != 3 && net->counters != nullptr &&
                               (chunks[i] == 2 || chunks[i] == 4) && counters_used + counters_need <= kTileCounters;
      if (fuse_reduce) {
        qs = q;                                // the layer keeps y, norm, residual, activation
        qs.parts = chunks[i];
        qs.kt_part = q.kt_chunk;
        qs.part_stride = r.part_stride;
        qs.part_buf = (float*)part_cur;
        qs.counters = net->counters + counters_used;
      }
      if (can_split && net->split_mode == 0) {
        const auto key = tune_key(q, 0, twins[i]);
        if (net->tuning && !net->tuned_split.count(key)) {
          // (a split layer is timed alone: copies of it would share its tile counters)
          float t_one = 0.f, t_split = 0.f;
          net->tuned[tune_key(q, 1, twins[i])] = measure_variants(q, true, nullptr, &t_one);
          net->tuned[tune_key(q, chunks[i], twins[i])] = measure_variants(qs, false, fuse_reduce ? nullptr : &r, &t_split);
          net->tuned_split[key] = t_split < t_one ? 1 : 0;
        }
        auto it = net->tuned_split.end();
        for (int tw = twins[i]; tw >= 1 && it == net->tuned_split.end(); --tw) it = net->tuned_split.find(tune_key(q, 0, tw));
        if (it != net->tuned_split.end()) split = it->second != 0;
      }
      if (split) {
        q = qs;
        if (fuse_reduce) counters_used += counters_need;
        else reduce.push_back(r);
        part_cur += part_bytes;
      }
      if (net->tuning && !net->tuned.count(tune_key(q, q.parts, twins[i]))) {
        float t = 0.f;
        net->tuned[tune_key(q, q.parts, twins[i])] = measure_variants(q, q.parts == 1 && chunks[i] > 1,
                                                                      (split && !fuse_reduce) ? &r : nullptr, &t,
                                                                      q.parts == 1 ? twins[i] : 1);
      }
      auto it = find_tuned(q, q.parts, twins[i]);
      if (it != net->tuned.end()) var[i] = it->second;
      if (net->forced_variant >= 0 && igemm_variant_ok(net->forced_variant, q)) var[i] = net->forced_variant;
      if (!igemm_variant_ok(var[i], q)) var[i] = pick_variant(q.M, q.K, q.C * q.R * q.S);
      place(q, var[i]);
    }
    if ((unify || n > 1) && !net->tuning) {
      // several problems in one slot (a mixed batch, or two layers sharing a launch): every extra tile
      // variant is an extra launch with its fixed cost, so there is one variant per kernel flavour,
      // that of the problem with the most work
      for (int chunked = 0; chunked < 2; ++chunked) {
        int lead = -1;
        double lead_work = -1;
        for (size_t i = 0; i < n; ++i) {
          if ((ps[i].parts == 1 && chunks[i] > 1) != (chunked == 1)) continue;
          const double work = (double)ps[i].M * ps[i].K * (ps[i].C * ps[i].R * ps[i].S + 64.0);
          if (work > lead_work) { lead_work = work; lead = (int)i; }
        }
        if (lead < 0) continue;
        for (size_t i = 0; i < n; ++i)
          if ((ps[i].parts == 1 && chunks[i] > 1) == (chunked == 1) && igemm_variant_ok(var[lead], ps[i])) {
            var[i] = var[lead];
            place(ps[i], var[i]);
          }
      }
    }
    if (err != hipSuccess) return;
    {
      size_t slot = 0;                       // counters of the reductions that finish inside the matrix launch
      for (size_t i = 0; i < n; ++i)
        if (ps[i].counters) {
          ps[i].counters = net->counters + slot;
          slot += (size_t)ps[i].tiles_base;
          if ((size_t)ps[i].parts * ps[i].part_stride > align_up((size_t)ps[i].parts * (ps[i].M + 128) * (ps[i].K + 192) * 4, 256)) {
            err = hipErrorInvalidValue;
            return;
          }
        }
      if (slot > kTileCounters) { err = hipErrorInvalidValue; return; }
    }
    for (int chunked = 0; chunked < 2; ++chunked)
      for (int v = 0; v < igemm_num_variants(); ++v) {
        ConvGroupArgs a;
        a.n = 0;
        int start = 0;
        double flops = 0, bytes = 0;
        for (size_t i = 0; i < n; ++i) {
          ConvProblem& p = ps[i];
          // one block walking several chunks folds them in registers: its own kernel instantiation
          const bool in_block_chunks = p.parts == 1 && chunks[i] > 1;
          if (var[i] != v || in_block_chunks != (chunked == 1)) continue;
          if (a.n == SNA_MAX_GROUPS) {       // more problems than one launch carries: flush
            a.total_tiles = start;
            emit(PlanOp::IGEMM, v, chunked, KC_IGEMM, flops, bytes, a);
            a.n = 0; start = 0; flops = 0; bytes = 0;
          }
          p.tile_start = start;
          start += p.tiles;
          a.p[a.n++] = p;
          const int cc = p.c_count ? p.c_count : p.C;     // channel padding is not algorithmic work
          const double mac = (double)p.M * p.K * cc * p.R * p.S;
          macs += (int64_t)mac;
          flops += 2 * mac;
          // algorithmic bytes of the layer (the split path's partial sums are overhead, not counted)
          bytes += 2.0 * ((double)p.N * p.H * p.W * cc + (double)p.K * p.R * p.S * cc) +
                   ((p.out_fp32 && (p.parts == 1 || p.counters)) ? 4.0 : 2.0) * (double)p.M * p.K + 8.0 * p.K +
                   (p.res ? 2.0 * p.M * p.K : 0.0);
        }
        a.total_tiles = start;
        if (a.n) emit(PlanOp::IGEMM, v, chunked, KC_IGEMM, flops, bytes, a);
      }
    for (size_t i = 0; i < reduce.size(); i += SNA_MAX_GROUPS) {
      ConvGroupArgs a;
      a.n = 0;
      int start = 0;
      for (size_t j = i; j < reduce.size() && j < i + SNA_MAX_GROUPS; ++j) {
        ConvProblem& r = reduce[j];
        r.tiles = (int)(((long)r.M * (r.K / 8) + 255) / 256);
        r.tile_start = start;
        start += r.tiles;
        a.p[a.n++] = r;
      }
      a.total_tiles = start;
      emit(PlanOp::KREDUCE, 0, 0, KC_KREDUCE, 0, 0, a);
    }
  }

  void run_direct(std::vector<ConvProblem>& ps) {
    if (ps.empty()) return;
    ConvGroupArgs a;
    a.n = 0;
    int start = 0;
    double flops = 0, bytes = 0;
    for (ConvProblem& p : ps) {
      p.tiles_n = (p.K + 15) / 16;
      p.tiles = ((p.M + 255) / 256) * p.tiles_n;
      p.tile_start = start;
      start += p.tiles;
      a.p[a.n++] = p;
      const double mac = (double)p.M * p.K * p.C * p.R * p.S;
      macs += (int64_t)mac;
      flops += 2 * mac;
      bytes += (double)esz() * ((double)p.N * p.H * p.W * p.C + (double)p.K * p.R * p.S * p.C) +
               (p.out_fp32 ? 4.0 : (double)esz()) * (double)p.M * p.K + 8.0 * p.K +
               (p.res ? (double)esz() * p.M * p.K : 0.0);
    }
    a.total_tiles = start;
    emit(PlanOp::DIRECT, 0, T().arch.dtype, KC_DIRECT, flops, bytes, a);
  }

  // ---- SubnetNorm calibration -----------------------------------------------------------------
  // Statistics-table rows behind a folded scale pointer: (subnet id, offset of the layer in a row).
  void norm_rows(const float* scale, NormCalArgs& c) const {
    const size_t rl = (size_t)T().row_len, idx = (size_t)(scale - net->folded);
    const size_t id = idx / (2 * rl), off = idx % (2 * rl);
    float* row = net->stats_mut + id * 4 * rl + off;
    c.mean = row; c.var = row + rl; c.gamma = row + 2 * rl; c.beta = row + 3 * rl;
    c.scale = net->folded + id * 2 * rl + off; c.shift = c.scale + rl;
  }
  // After the raw fp32 output of a layer is in `raw`: measure it, store the statistics, normalise.
  void calibrate_layer(const float* raw, float* part, int M, int K, const float* scale, const void* res, void* y,
                       int act, int res_after_act, int res_stride, int y_stride) {
    NormCalArgs c;
    memset(&c, 0, sizeof(c));
    c.raw = raw; c.M = M; c.K = K; c.part = part; c.nrb = (M + SNA_CAL_ROWS - 1) / SNA_CAL_ROWS;
    norm_rows(scale, c);
    emit(PlanOp::NORMCAL, 0, 0, KC_CALIB, 0, 4.0 * M * K, c);
    NormApplyArgs ap;
    memset(&ap, 0, sizeof(ap));
    ap.raw = raw; ap.scale = c.scale; ap.shift = c.shift; ap.res = res; ap.y = y;
    ap.M = M; ap.K = K; ap.act = act; ap.res_after_act = res_after_act; ap.res_stride = res_stride; ap.y_stride = y_stride;
    emit(PlanOp::NORMAPPLY, 0, T().arch.dtype, KC_CALIB, 0, (4.0 + 2.0 * esz()) * M * K, ap);
  }
  // Room for a layer's raw output and its row-block partials in the fp32 scratch region (which the
  // split reductions, switched off while calibrating, otherwise use).
  bool cal_scratch(char*& cur, int M, int K, float*& raw, float*& part) {
    const size_t raw_b = align_up((size_t)M * K * 4, 256);
    const size_t part_b = align_up((size_t)((M + SNA_CAL_ROWS - 1) / SNA_CAL_ROWS) * K * 3 * 4, 256);
    if ((size_t)(cur - net->partials) + raw_b + part_b > net->partials_bytes) { err = hipErrorOutOfMemory; return false; }
    raw = (float*)cur; part = (float*)(cur + raw_b);
    cur += raw_b + part_b;
    return true;
  }
  // A conv slot while calibrating: layers with SubnetNorm run bare (no scale / shift / activation /
  // residual, fp32 output), then each is measured and normalised; the others run as usual.
  void calibrate_convs(std::vector<ConvProblem>& ps, bool direct) {
    std::vector<ConvProblem> plain, bare, orig;
    char* cur = net->partials;
    std::vector<std::pair<float*, float*>> bufs;
    for (ConvProblem& p : ps) {
      if (!p.scale) { plain.push_back(p); continue; }
      float *raw, *part;
      if (!cal_scratch(cur, p.M, p.K, raw, part)) return;
      orig.push_back(p);
      ConvProblem b = p;
      b.scale = nullptr; b.shift = nullptr; b.res = nullptr; b.act = SNA_ACT_NONE; b.res_after_act = 0;
      b.y = raw; b.y_stride = p.K; b.out_fp32 = 1;
      bare.push_back(b);
      bufs.push_back({raw, part});
    }
    if (direct) { run_direct(plain); run_direct(bare); } else { run_igemm(plain); run_igemm(bare); }
    for (size_t i = 0; i < orig.size(); ++i) {
      const ConvProblem& p = orig[i];
      calibrate_layer(bufs[i].first, bufs[i].second, p.M, p.K, p.scale, p.res, p.y, p.act, p.res_after_act, p.res_stride,
                      p.y_stride);
    }
  }

  // One conv slot over all groups.  `fill` returns false for groups that skip the slot.
  void conv_slot(bool direct, const std::function<bool(Group&, ConvProblem&)>& fill) {
    std::vector<ConvProblem> ps;
    for (Group& g : groups) {
      ConvProblem p;
      memset(&p, 0, sizeof(p));
      if (fill(g, p)) ps.push_back(p);
    }
    if (net->calibrating) { calibrate_convs(ps, direct); return; }
    if (direct) run_direct(ps); else run_igemm(ps);
  }

  // Two layers that read the same input and do not depend on each other (a stage's conv1 and its
  // projection shortcut) go into one grouped launch: they share one tile variant, the one chosen for
  // the layer with more work, and the second launch with its fixed cost disappears.
  void conv_slot2(const std::function<bool(Group&, ConvProblem&)>& fill_a,
                  const std::function<bool(Group&, ConvProblem&)>& fill_b) {
    std::vector<ConvProblem> ps;
    for (int which = 0; which < 2; ++which)
      for (Group& g : groups) {
        ConvProblem p;
        memset(&p, 0, sizeof(p));
        if ((which == 0 ? fill_a : fill_b)(g, p)) ps.push_back(p);
      }
    if (net->calibrating) { calibrate_convs(ps, false); return; }
    if (ps.size() > SNA_MAX_GROUPS) {      // would not fit one launch anyway
      std::vector<ConvProblem> a(ps.begin(), ps.begin() + ps.size() / 2), b(ps.begin() + ps.size() / 2, ps.end());
      run_igemm(a);
      run_igemm(b);
      return;
    }
    run_igemm(ps, true);
  }


  void pool_slot(bool is_max, const std::function<bool(Group&, PoolProblem&)>& fill) {
    PoolGroupArgs a;
    a.n = 0;
    int start = 0;
    double bytes = 0;
    for (Group& g : groups) {
      PoolProblem p;
      memset(&p, 0, sizeof(p));
      if (!fill(g, p)) continue;
      if (is_max) {
        p.Ho = out_size(p.H, 3, 2); p.Wo = out_size(p.W, 3, 2);
        const long total = (long)p.N * p.Ho * p.Wo * (p.C / 8);
        p.tiles = (int)((total + 255) / 256);
      } else {
        p.Ho = p.Wo = 1;
        p.tiles = p.N * ((p.C / 8 + 31) / 32);
      }
      p.tile_start = start;
      start += p.tiles;
      bytes += (double)esz() * ((double)p.N * p.H * p.W * p.C + (double)p.N * p.Ho * p.Wo * p.C);
      a.p[a.n++] = p;
    }
    if (!a.n) return;
    const int dt = T().arch.dtype;
    if (is_max) emit(PlanOp::MAXPOOL, 0, dt, KC_POOL, 0, bytes, a);
    else emit(PlanOp::GAP, 0, dt, KC_POOL, 0, bytes, a);
  }

  void dw_slot(const std::function<bool(Group&, DwProblem&)>& fill) {
    DwGroupArgs a;
    a.n = 0;
    double flops = 0, bytes = 0;
    for (Group& g : groups) {
      DwProblem p;
      memset(&p, 0, sizeof(p));
      if (!fill(g, p)) continue;
      flops += 2.0 * p.N * p.Ho * p.Wo * p.C * p.k * p.k;
      macs += (int64_t)p.N * p.Ho * p.Wo * p.C * p.k * p.k;
      bytes += 2.0 * p.N * p.C * ((double)p.H * p.W + (double)p.Ho * p.Wo) + 2.0 * p.k * p.k * p.C + 8.0 * p.C;
      a.p[a.n++] = p;
    }
    if (!a.n) return;
    if (!net->calibrating) { emit(PlanOp::DW, 0, 0, KC_DEPTHWISE, flops, bytes, a); return; }
    // calibration: bare fp32 sums first, then statistics and the normalise pass per layer
    DwGroupArgs bare = a;
    char* cur = net->partials;
    std::vector<std::pair<float*, float*>> bufs;
    for (int i = 0; i < a.n; ++i) {
      float *raw, *part;
      if (!cal_scratch(cur, a.p[i].N * a.p[i].Ho * a.p[i].Wo, a.p[i].C, raw, part)) return;
      bare.p[i].y = raw; bare.p[i].raw_out = 1; bare.p[i].pool_part = nullptr; bare.p[i].bpr = 0;
      bufs.push_back({raw, part});
    }
    emit(PlanOp::DW, 0, 0, KC_DEPTHWISE, flops, bytes, bare);
    for (int i = 0; i < a.n; ++i)
      calibrate_layer(bufs[i].first, bufs[i].second, a.p[i].N * a.p[i].Ho * a.p[i].Wo, a.p[i].C, a.p[i].scale, nullptr,
                      a.p[i].y, a.p[i].act, 0, a.p[i].C, a.p[i].C);
  }
  // Depthwise WeightSlice: leading C channels, centre k x k window of the stored kernel.
  void slice_dw(DwProblem& p, const sna_tensor_info& ti, int k, int stride) {
    const int rmax = ti.dims[0], smax = ti.dims[1], cmax = ti.dims[2];
    p.wr = smax * cmax; p.ws = cmax;
    const int r0 = (rmax - k) / 2, s0 = (smax - k) / 2;
    p.w = wptr(ti) + ((size_t)r0 * p.wr + (size_t)s0 * p.ws) * 2;
    p.k = k; p.stride = stride; p.pad = k / 2;
    p.Ho = out_size(p.H, k, stride); p.Wo = out_size(p.W, k, stride);
  }
  void se_slot(const std::function<bool(Group&, SeProblem&)>& fill) {
    SeGroupArgs a;
    a.n = 0;
    double flops = 0, bytes = 0;
    for (Group& g : groups) {
      SeProblem p;
      memset(&p, 0, sizeof(p));
      if (!fill(g, p)) continue;
      flops += 4.0 * p.N * p.C * p.Q;
      macs += (int64_t)2 * p.N * p.C * p.Q;
      bytes += 4.0 * p.N * p.HW * p.C + 4.0 * p.C * p.Q;
      a.p[a.n++] = p;
    }
    if (a.n) emit(PlanOp::SE, 0, 0, KC_SE, flops, bytes, a);
  }

  // ---- request gather / logits scatter -----------------------------------------------------
  void copy_items(const void* src, void* dst, std::vector<CopyItem>& items) {
    for (size_t i = 0; i < items.size(); i += SNA_COPY_ITEMS) {
      CopyArgs a;
      a.src = src; a.dst = dst;
      a.n = (int)std::min<size_t>(SNA_COPY_ITEMS, items.size() - i);
      double bytes = 0;
      for (int j = 0; j < a.n; ++j) { a.it[j] = items[i + j]; bytes += 2.0 * items[i + j].n; }
      emit(PlanOp::COPY, 0, 0, KC_COPY, 0, bytes, a);
    }
  }

  // ResNet family: 7x7 stem conv + SubnetNorm + ReLU + max pool as one kernel (which also reads unpadded images)
  bool resnet_fused_stem() const {
    const sna_arch_desc& a = T().arch;
    bool fused = a.dtype == SNA_DTYPE_BF16 && a.in_ch == 3 && tensor("stem.w").dims[1] == 7 && tensor("stem.w").dims[2] == 7;
    for (const Group& g : groups) fused = fused && g.cfg->stage_out_ch[0] <= 64;
    return fused && !net->calibrating;     // calibration needs the stem's bare output
  }
  // MBV3 family: stem + fixed first block as one kernel (which also reads unpadded images)
  bool mbv3_fused_head() const {
    const sna_arch_desc& a = T().arch;
    const sna_tensor_info& ws = tensor("stem.w");
    const sna_tensor_info& wd = tensor("first.dw.w");
    return a.dtype == SNA_DTYPE_BF16 && a.in_ch == 3 && a.stem_ch == mbv3_head_channels() && ws.dims[1] == 3 && ws.dims[2] == 3 &&
           wd.dims[0] >= 3 && wd.dims[1] >= 3 && !net->calibrating;     // calibration needs every layer's bare output
  }
  sna_status run_tiny(const void* inputs, float* logits);
  sna_status run_resnet(const void* inputs, float* logits);
  sna_status run_mbv3(const void* inputs, float* logits);
  sna_status run_transformer(const void* inputs, float* logits, void* hidden);

  // Point every group at its requests' inputs: in place when they are contiguous in the call,
  // otherwise gathered into the group's input buffer.
  void bind_inputs(const void* inputs, const std::vector<size_t>& req_off, const std::vector<size_t>& req_bytes) {
    std::vector<CopyItem> items;
    for (Group& g : groups) {
      if (g.contiguous) {
        g.cur = (const char*)inputs + req_off[g.reqs[0]];
      } else {
        size_t d = 0;
        for (int r : g.reqs) {
          items.push_back({req_off[r], (size_t)(g.inbuf - net->arena) + d, req_bytes[r]});
          d += req_bytes[r];
        }
        g.cur = g.inbuf;
      }
    }
    if (!items.empty()) copy_items(inputs, net->arena, items);
  }

  // bf16 image families: every group's requests are copied into its input buffer with the
  // channels padded to 8 (which also gathers scattered requests), so the stem runs on MFMA.
  void pad_inputs(const void* inputs, const std::vector<size_t>& req_off, bool raw_ok) {
    const int c_in = T().arch.in_ch;
    std::vector<PadItem> items;
    for (Group& g : groups) {
      if (raw_ok && g.contiguous) {        // the first layer reads the caller's images in place
        g.cur = (const char*)inputs + req_off[g.reqs[0]];
        g.raw_input = true;
        continue;
      }
      const size_t pix = (size_t)g.cfg->in_h * g.cfg->in_w;
      size_t d = (size_t)(g.inbuf - net->arena);
      if (g.contiguous) {
        items.push_back({req_off[g.reqs[0]], d, pix * g.n});
      } else {
        for (int r : g.reqs) { items.push_back({req_off[r], d, pix}); d += pix * 16; }
      }
      g.cur = g.inbuf;
    }
    for (size_t i = 0; i < items.size(); i += SNA_PAD_ITEMS) {
      PadArgs a;
      a.src = inputs; a.dst = net->arena; a.c_in = c_in;
      a.n = (int)std::min<size_t>(SNA_PAD_ITEMS, items.size() - i);
      double bytes = 0;
      for (int j = 0; j < a.n; ++j) { a.it[j] = items[i + j]; bytes += (2.0 * c_in + 16.0) * items[i + j].pixels; }
      emit(PlanOp::PAD, 0, 0, KC_COPY, 0, bytes, a);
    }
  }

  // The head writes logits straight to the caller's buffer for contiguous groups, else into
  // the group's scratch; scatter_logits() then moves rows to request order.
  float* logits_target(Group& g, float* logits) {
    const int nc = T().arch.n_classes;
    return g.contiguous ? logits + (size_t)g.reqs[0] * nc : g.small;
  }
  void scatter_logits(float* logits) {
    const int nc = T().arch.n_classes;
    for (Group& g : groups) {
      if (g.contiguous) continue;
      std::vector<CopyItem> items;
      for (int i = 0; i < g.n; ++i)
        items.push_back({(size_t)i * nc * 4, (size_t)g.reqs[i] * nc * 4, (size_t)nc * 4});
      copy_items(g.small, logits, items);
    }
  }
};

// ------------------------------------------------------------------------------------------
// TINY: stem 3x3 -> SN -> ReLU; blocks conv3x3 -> SN -> ReLU (+ residual for j >= 1); GAP; linear
// ------------------------------------------------------------------------------------------
sna_status Fwd::run_tiny(const void*, float* logits) {
  const sna_arch_desc& a = T().arch;
  for (Group& g : groups) { g.H = g.cfg->in_h; g.W = g.cfg->in_w; g.C = a.in_ch; }
  auto conv = [&](const std::string& wname, const std::string& nname, int stride, bool residual,
                  const std::function<bool(const Group&)>& active, const std::function<int(const Group&)>& kout) {
    conv_slot(true, [&](Group& g, ConvProblem& p) {
      if (!active(g)) return false;
      p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
      slice_conv(p, tensor(wname), kout(g), 3, stride);
      p.scale = scale_of(nname, g.cfg->subnet_id); p.shift = shift_of(nname, g.cfg->subnet_id);
      p.act = SNA_ACT_RELU;
      const int dst = g.cur_buf == 0 ? 1 : 0;
      p.y = g.buf[dst];
      if (residual) { p.res = g.cur; p.res_after_act = 1; }
      g.cur = p.y; g.cur_buf = dst; g.H = p.Ho; g.W = p.Wo; g.C = p.K;
      return true;
    });
  };
  conv("stem.w", "stem.sn", 1, false, [](const Group&) { return true; },
       [&](const Group& g) { return g.cfg->stage_out_ch[0]; });
  for (int s = 0; s < a.n_stages; ++s)
    for (int j = 0; j < a.stage_max_depth[s]; ++j) {
      const std::string p = "s" + std::to_string(s) + ".b" + std::to_string(j) + ".";
      conv(p + "w", p + "sn", j == 0 ? 2 : 1, j > 0, [&](const Group& g) { return j < g.cfg->depth[s]; },
           [&](const Group& g) { return g.cfg->stage_out_ch[1 + s]; });
    }
  pool_slot(false, [&](Group& g, PoolProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
    p.y = g.buf[2];
    g.cur = p.y; g.H = g.W = 1;
    return true;
  });
  conv_slot(true, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = 1; p.W = 1; p.C = g.C;
    slice_conv(p, tensor("head.w"), a.n_classes, 1, 1);
    p.shift = (const float*)wptr(tensor("head.b"));
    p.y = logits_target(g, logits); p.out_fp32 = 1;
    return true;
  });
  scatter_logits(logits);
  return SNA_OK;
}

// ------------------------------------------------------------------------------------------
// RESNET bottleneck SuperNet
// ------------------------------------------------------------------------------------------
sna_status Fwd::run_resnet(const void*, float* logits) {
  const sna_arch_desc& a = T().arch;
  for (Group& g : groups) { g.H = g.cfg->in_h; g.W = g.cfg->in_w; g.C = 8; }     // channel-padded inputs
  const bool fused_stem = resnet_fused_stem();
  if (fused_stem) {
    // stem conv + SubnetNorm + ReLU + max pool in one kernel: the conv output stays in LDS
    StemPoolArgs sa;
    sa.n = 0;
    int start = 0;
    double flops = 0, bytes = 0;
    for (Group& g : groups) {
      ConvProblem c;
      memset(&c, 0, sizeof(c));
      c.N = g.n; c.H = g.H; c.W = g.W; c.C = g.C;
      slice_conv(c, tensor("stem.w"), g.cfg->stage_out_ch[0], 7, 2);
      StemPoolProblem p;
      memset(&p, 0, sizeof(p));
      p.x = g.cur; p.w = c.w; p.y = g.buf[1];
      p.scale = scale_of("stem.sn", g.cfg->subnet_id); p.shift = shift_of("stem.sn", g.cfg->subnet_id);
      p.N = g.n; p.H = g.H; p.W = g.W; p.Ho = c.Ho; p.Wo = c.Wo;
      p.Po = out_size(c.Ho, 3, 2); p.Qo = out_size(c.Wo, 3, 2);
      p.K = c.K; p.wk = c.wk; p.wr = c.wr; p.ws = c.ws;
      p.pix_b = g.raw_input ? 2 * a.in_ch : 16;
      p.x_bytes = (unsigned)((size_t)g.n * g.H * g.W * p.pix_b);
      p.tiles_x = (p.Qo + 15) / 16; p.tiles_y = (p.Po + 3) / 4;
      p.tiles = p.N * p.tiles_x * p.tiles_y;
      p.tile_start = start;
      start += p.tiles;
      sa.p[sa.n++] = p;
      const double mac = (double)c.M * c.K * a.in_ch * 49;        // channel padding is not algorithmic work
      macs += (int64_t)mac;
      flops += 2 * mac;
      bytes += 2.0 * ((double)g.n * g.H * g.W * a.in_ch + (double)c.K * 49 * a.in_ch) + 8.0 * c.K +
               2.0 * (double)g.n * p.Po * p.Qo * c.K;
      g.cur = p.y; g.cur_buf = 1; g.H = p.Po; g.W = p.Qo; g.C = c.K;
    }
    sa.total_tiles = start;
    emit(PlanOp::STEMPOOL, 0, 0, KC_STEMPOOL, flops, bytes, sa);
  } else {
    conv_slot(false, [&](Group& g, ConvProblem& p) {
      p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
      slice_conv(p, tensor("stem.w"), g.cfg->stage_out_ch[0], 7, 2);
      p.c_count = a.in_ch;
      p.scale = scale_of("stem.sn", g.cfg->subnet_id); p.shift = shift_of("stem.sn", g.cfg->subnet_id);
      p.act = SNA_ACT_RELU; p.y = g.buf[0];
      g.cur = p.y; g.cur_buf = 0; g.H = p.Ho; g.W = p.Wo; g.C = p.K;
      return true;
    });
    pool_slot(true, [&](Group& g, PoolProblem& p) {
      p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C; p.y = g.buf[1];
      g.cur = p.y; g.cur_buf = 1; g.H = out_size(g.H, 3, 2); g.W = out_size(g.W, 3, 2);
      return true;
    });
  }
  // buffers: block input lives in buf[0] or buf[1]; buf[2] conv1 out, buf[3] conv2 out, buf[4] shortcut
  for (int s = 0; s < a.n_stages; ++s)
    for (int j = 0; j < a.stage_max_depth[s]; ++j) {
      const std::string pre = "s" + std::to_string(s) + ".b" + std::to_string(j) + ".";
      const int st = j == 0 ? a.stage_stride[s] : 1;
      auto on = [&](const Group& g) { return j < g.cfg->depth[s]; };
      auto conv1 = [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
        slice_conv(p, tensor(pre + "conv1.w"), g.cfg->block_mid_ch[s][j], 1, 1);
        p.scale = scale_of(pre + "sn1", g.cfg->subnet_id); p.shift = shift_of(pre + "sn1", g.cfg->subnet_id);
        p.act = SNA_ACT_RELU; p.y = g.buf[2];
        return true;
      };
      auto shortcut = [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
        slice_conv(p, tensor(pre + "short.w"), g.cfg->stage_out_ch[1 + s], 1, st);
        p.scale = scale_of(pre + "sn_short", g.cfg->subnet_id);
        p.shift = shift_of(pre + "sn_short", g.cfg->subnet_id);
        p.act = SNA_ACT_NONE; p.y = g.buf[4];
        return true;
      };
      if (j == 0) conv_slot2(conv1, shortcut);
      else conv_slot(false, conv1);
      conv_slot(false, [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        const int m = g.cfg->block_mid_ch[s][j];
        p.x = g.buf[2]; p.N = g.n; p.H = g.H; p.W = g.W; p.C = m;
        slice_conv(p, tensor(pre + "conv2.w"), m, 3, st);
        p.scale = scale_of(pre + "sn2", g.cfg->subnet_id); p.shift = shift_of(pre + "sn2", g.cfg->subnet_id);
        p.act = SNA_ACT_RELU; p.y = g.buf[3];
        return true;
      });
      conv_slot(false, [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        const int m = g.cfg->block_mid_ch[s][j];
        p.x = g.buf[3]; p.N = g.n; p.H = out_size(g.H, 3, st); p.W = out_size(g.W, 3, st); p.C = m;
        slice_conv(p, tensor(pre + "conv3.w"), g.cfg->stage_out_ch[1 + s], 1, 1);
        p.scale = scale_of(pre + "sn3", g.cfg->subnet_id); p.shift = shift_of(pre + "sn3", g.cfg->subnet_id);
        p.act = SNA_ACT_RELU;
        p.res = j == 0 ? (const void*)g.buf[4] : g.cur; p.res_after_act = 0;
        const int dst = g.cur_buf == 0 ? 1 : 0;
        p.y = g.buf[dst];
        g.cur = p.y; g.cur_buf = dst; g.H = p.H; g.W = p.W; g.C = p.K;
        return true;
      });
    }
  pool_slot(false, [&](Group& g, PoolProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C; p.y = g.buf[2];
    g.cur = p.y; g.H = g.W = 1;
    return true;
  });
  conv_slot(a.n_classes % 8 != 0, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = 1; p.W = 1; p.C = g.C;
    slice_conv(p, tensor("head.w"), a.n_classes, 1, 1);
    p.shift = (const float*)wptr(tensor("head.b"));
    p.y = logits_target(g, logits); p.out_fp32 = 1;
    return true;
  });
  scatter_logits(logits);
  return SNA_OK;
}

// ------------------------------------------------------------------------------------------
// MBV3-shaped SuperNet: stem, fixed depthwise-separable block, inverted-residual stages, head
// ------------------------------------------------------------------------------------------
sna_status Fwd::run_mbv3(const void*, float* logits) {
  const sna_arch_desc& a = T().arch;
  for (Group& g : groups) { g.H = g.cfg->in_h; g.W = g.cfg->in_w; g.C = 8; }     // channel-padded inputs
  auto sn = [&](ConvProblem& p, const std::string& name, const Group& g) {
    p.scale = scale_of(name, g.cfg->subnet_id); p.shift = shift_of(name, g.cfg->subnet_id);
  };
  if (mbv3_fused_head()) {
    Mbv3HeadArgs ha;
    ha.n = 0;
    double flops = 0, bytes = 0;
    auto flush = [&] {
      if (ha.n) emit(PlanOp::MBV3HEAD, 0, 0, KC_STEMPOOL, flops, bytes, ha);
      ha.n = 0; flops = 0; bytes = 0;
    };
    for (Group& g : groups) {
      ConvProblem c, pw;
      memset(&c, 0, sizeof(c));
      c.N = g.n; c.H = g.H; c.W = g.W; c.C = g.C;
      slice_conv(c, tensor("stem.w"), a.stem_ch, 3, 2);
      DwProblem d;
      memset(&d, 0, sizeof(d));
      d.N = g.n; d.H = c.Ho; d.W = c.Wo; d.C = a.stem_ch;
      slice_dw(d, tensor("first.dw.w"), 3, 1);
      memset(&pw, 0, sizeof(pw));
      pw.N = g.n; pw.H = c.Ho; pw.W = c.Wo; pw.C = a.stem_ch;
      slice_conv(pw, tensor("first.pw.w"), a.stem_ch, 1, 1);
      Mbv3HeadProblem p;
      memset(&p, 0, sizeof(p));
      p.x = g.cur; p.y = g.buf[1];
      p.w_stem = c.w; p.wk0 = c.wk; p.wr0 = c.wr; p.ws0 = c.ws;
      p.w_dw = d.w; p.wr1 = d.wr; p.ws1 = d.ws;
      p.w_pw = pw.w; p.wk2 = pw.wk;
      p.sc0 = scale_of("stem.sn", g.cfg->subnet_id); p.sh0 = shift_of("stem.sn", g.cfg->subnet_id);
      p.sc1 = scale_of("first.sn1", g.cfg->subnet_id); p.sh1 = shift_of("first.sn1", g.cfg->subnet_id);
      p.sc2 = scale_of("first.sn2", g.cfg->subnet_id); p.sh2 = shift_of("first.sn2", g.cfg->subnet_id);
      p.N = g.n; p.H = g.H; p.W = g.W; p.Ho = c.Ho; p.Wo = c.Wo;
      p.pix_e = g.raw_input ? a.in_ch : 8;
      const double px = (double)g.n * c.Ho * c.Wo, mac = px * a.stem_ch * (9.0 * a.in_ch + 9.0 + a.stem_ch);
      macs += (int64_t)mac;
      flops += 2 * mac;
      bytes += 2.0 * ((double)g.n * g.H * g.W * a.in_ch + px * a.stem_ch) +
               2.0 * a.stem_ch * (9.0 * a.in_ch + 9.0 + a.stem_ch) + 24.0 * a.stem_ch;
      if (ha.n == SNA_MAX_GROUPS) flush();
      ha.p[ha.n++] = p;
      g.cur = p.y; g.cur_buf = 1; g.H = c.Ho; g.W = c.Wo; g.C = a.stem_ch;
    }
    flush();
  } else {
  conv_slot(false, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
    slice_conv(p, tensor("stem.w"), a.stem_ch, 3, 2);
    p.c_count = a.in_ch;
    sn(p, "stem.sn", g);
    p.act = SNA_ACT_HSWISH; p.y = g.buf[0];
    g.cur = p.y; g.cur_buf = 0; g.H = p.Ho; g.W = p.Wo; g.C = p.K;
    return true;
  });
  // fixed first block: depthwise 3x3 + SN + ReLU -> 1x1 + SN, residual
  dw_slot([&](Group& g, DwProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
    slice_dw(p, tensor("first.dw.w"), 3, 1);
    p.scale = scale_of("first.sn1", g.cfg->subnet_id); p.shift = shift_of("first.sn1", g.cfg->subnet_id);
    p.act = SNA_ACT_RELU; p.y = g.buf[2];
    return true;
  });
  conv_slot(false, [&](Group& g, ConvProblem& p) {
    p.x = g.buf[2]; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
    slice_conv(p, tensor("first.pw.w"), a.stem_ch, 1, 1);
    sn(p, "first.sn2", g);
    p.act = SNA_ACT_NONE; p.res = g.cur; p.y = g.buf[1];
    g.cur = p.y; g.cur_buf = 1;
    return true;
  });
  }
  for (int s = 0; s < a.n_stages; ++s)
    for (int j = 0; j < a.stage_max_depth[s]; ++j) {
      const std::string pre = "s" + std::to_string(s) + ".b" + std::to_string(j) + ".";
      const int st = j == 0 ? a.stage_stride[s] : 1;
      const int act = a.stage_act[s];
      auto on = [&](const Group& g) { return j < g.cfg->depth[s]; };      // LayerSelect
      conv_slot(false, [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
        slice_conv(p, tensor(pre + "expand.w"), g.cfg->block_mid_ch[s][j], 1, 1);
        sn(p, pre + "sn1", g);
        p.act = act; p.y = g.buf[2];
        return true;
      });
      dw_slot([&](Group& g, DwProblem& p) {
        if (!on(g)) return false;
        p.x = g.buf[2]; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.cfg->block_mid_ch[s][j];
        slice_dw(p, tensor(pre + "dw.w"), g.cfg->block_kernel[s][j], st);
        p.scale = scale_of(pre + "sn2", g.cfg->subnet_id); p.shift = shift_of(pre + "sn2", g.cfg->subnet_id);
        p.act = act; p.y = g.buf[3];
        if (a.stage_se[s] && !net->calibrating) {               // the gate's average pool rides on this launch
          p.pool_part = g.small;
          p.bpr = depthwise_pool_blocks(p.Ho, p.Wo, p.C);
        }
        return true;
      });
      if (a.stage_se[s]) {
        if (net->calibrating)                                  // the pool could not ride on a bare-output launch
          pool_slot(false, [&](Group& g, PoolProblem& p) {
            if (!on(g)) return false;
            p.x = g.buf[3]; p.N = g.n; p.H = out_size(g.H, 3, st); p.W = out_size(g.W, 3, st);
            p.C = g.cfg->block_mid_ch[s][j]; p.y = g.small; p.out_fp32 = 1;
            return true;
          });
        se_slot([&](Group& g, SeProblem& p) {
          if (!on(g)) return false;
          const int m = g.cfg->block_mid_ch[s][j];
          const sna_tensor_info& t1 = tensor(pre + "se.fc1.w");
          const sna_tensor_info& t2 = tensor(pre + "se.fc2.w");
          p.x = g.buf[3]; p.y = g.buf[3];
          p.w1 = wptr(t1); p.b1 = (const float*)wptr(tensor(pre + "se.fc1.b")); p.w1_stride = t1.dims[1];
          p.w2 = wptr(t2); p.b2 = (const float*)wptr(tensor(pre + "se.fc2.b")); p.w2_stride = t2.dims[1];
          const int ho = out_size(g.H, 3, st), wo = out_size(g.W, 3, st);
          p.N = g.n; p.HW = ho * wo; p.C = m; p.Q = g.cfg->block_aux_ch[s][j];
          p.pool_segs = depthwise_pool_blocks(ho, wo, m); p.inv_hw = 1.f / (float)p.HW;
          if (net->calibrating) { p.pool_segs = 1; p.inv_hw = 1.f; }      // g.small holds the mean itself
          p.pooled = g.small;                                  // written by the depthwise launch above
          p.hidden = g.small + (size_t)p.pool_segs * g.n * m;
          return true;
        });
      }
      conv_slot(false, [&](Group& g, ConvProblem& p) {
        if (!on(g)) return false;
        const int co = a.stage_ch[s];
        p.x = g.buf[3]; p.N = g.n; p.H = out_size(g.H, 3, st); p.W = out_size(g.W, 3, st);
        p.C = g.cfg->block_mid_ch[s][j];
        slice_conv(p, tensor(pre + "project.w"), co, 1, 1);
        sn(p, pre + "sn3", g);
        p.act = SNA_ACT_NONE;
        if (st == 1 && g.C == co) p.res = g.cur;
        const int dst = g.cur_buf == 0 ? 1 : 0;
        p.y = g.buf[dst];
        g.cur = p.y; g.cur_buf = dst; g.H = p.H; g.W = p.W; g.C = co;
        return true;
      });
    }
  conv_slot(false, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C;
    slice_conv(p, tensor("tail.w"), a.tail_ch, 1, 1);
    sn(p, "tail.sn", g);
    p.act = SNA_ACT_HSWISH; p.y = g.buf[2];
    g.cur = p.y; g.C = a.tail_ch;
    return true;
  });
  pool_slot(false, [&](Group& g, PoolProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = g.H; p.W = g.W; p.C = g.C; p.y = g.buf[3];
    g.cur = p.y; g.H = g.W = 1;
    return true;
  });
  conv_slot(false, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = 1; p.W = 1; p.C = g.C;
    slice_conv(p, tensor("fc1.w"), a.fc_ch, 1, 1);
    p.shift = (const float*)wptr(tensor("fc1.b"));
    p.act = SNA_ACT_HSWISH; p.y = g.buf[4];
    g.cur = p.y; g.C = a.fc_ch;
    return true;
  });
  conv_slot(a.n_classes % 8 != 0, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = 1; p.W = 1; p.C = g.C;
    slice_conv(p, tensor("head.w"), a.n_classes, 1, 1);
    p.shift = (const float*)wptr(tensor("head.b"));
    p.y = logits_target(g, logits); p.out_fp32 = 1;
    return true;
  });
  scatter_logits(logits);
  return SNA_OK;
}
// ------------------------------------------------------------------------------------------
// TRANSFORMER: post-LayerNorm encoder layers; leading heads / leading FFN columns per layer
// ------------------------------------------------------------------------------------------
sna_status Fwd::run_transformer(const void*, float* logits, void* hidden) {
  const sna_arch_desc& a = T().arch;
  const int hd = a.hidden, S = a.seq_len;
  // buffers: x in buf[0] / buf[1] (or the caller's input), q k v ctx u ffn in buf[2..7]
  auto linear = [&](Group& g, ConvProblem& p, const void* x, int c_in, const std::string& w, int n_out,
                    const std::string& bias, int act, const void* res, void* y) {
    memset(&p, 0, sizeof(p));
    p.x = x; p.N = g.n * S; p.H = 1; p.W = 1; p.C = c_in;
    slice_conv(p, tensor(w), n_out, 1, 1);
    p.shift = (const float*)wptr(tensor(bias));
    p.act = act; p.res = res; p.y = y;
  };
  auto layernorm = [&](const std::string& gname, const std::string& bname, int j, int src, bool to_cur_other) {
    LnGroupArgs la;
    la.n = 0;
    double bytes = 0;
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;
      LnProblem p;
      memset(&p, 0, sizeof(p));
      p.x = g.buf[src];
      p.gamma = (const float*)wptr(tensor(gname)); p.beta = (const float*)wptr(tensor(bname));
      const int dst = g.cur_buf == 0 ? 1 : 0;
      p.y = g.buf[dst];
      p.rows = g.n * S; p.cols = hd;
      g.cur = p.y; g.cur_buf = dst;
      bytes += 4.0 * p.rows * p.cols + 8.0 * p.cols;
      la.p[la.n++] = p;
    }
    (void)to_cur_other;
    if (la.n) emit(PlanOp::LN, 0, 0, KC_LAYERNORM, 0, bytes, la);
  };
  for (int j = 0; j < a.max_layers; ++j) {
    const std::string pre = "l" + std::to_string(j) + ".";
    std::vector<ConvProblem> ps;
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;                 // LayerSelect
      const int at = g.cfg->block_mid_ch[0][j];
      ConvProblem p;
      linear(g, p, g.cur, hd, pre + "q.w", at, pre + "q.b", SNA_ACT_NONE, nullptr, g.buf[2]); ps.push_back(p);
      linear(g, p, g.cur, hd, pre + "k.w", at, pre + "k.b", SNA_ACT_NONE, nullptr, g.buf[3]); ps.push_back(p);
      linear(g, p, g.cur, hd, pre + "v.w", at, pre + "v.b", SNA_ACT_NONE, nullptr, g.buf[4]); ps.push_back(p);
    }
    if (ps.empty()) continue;
    run_igemm(ps);
    AttnGroupArgs aa;
    aa.n = 0;
    double aflops = 0, abytes = 0;
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;
      const int at = g.cfg->block_mid_ch[0][j];
      AttnProblem p;
      memset(&p, 0, sizeof(p));
      p.q = g.buf[2]; p.k = g.buf[3]; p.v = g.buf[4]; p.o = g.buf[5];
      p.B = g.n; p.S = S; p.heads = at / a.head_dim; p.ld = at;
      aflops += 4.0 * p.B * p.heads * S * S * a.head_dim;
      macs += (int64_t)2 * p.B * p.heads * S * S * a.head_dim;
      abytes += 2.0 * 4 * p.B * S * at;
      aa.p[aa.n++] = p;
    }
    emit(PlanOp::ATTN, 0, 0, KC_ATTENTION, aflops, abytes, aa);
    ps.clear();
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;
      ConvProblem p;
      linear(g, p, g.buf[5], g.cfg->block_mid_ch[0][j], pre + "o.w", hd, pre + "o.b", SNA_ACT_NONE, g.cur, g.buf[6]);
      ps.push_back(p);
    }
    run_igemm(ps);
    layernorm(pre + "ln1.g", pre + "ln1.b", j, 6, true);
    ps.clear();
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;
      ConvProblem p;
      linear(g, p, g.cur, hd, pre + "ffn1.w", g.cfg->block_aux_ch[0][j], pre + "ffn1.b", SNA_ACT_GELU, nullptr, g.buf[7]);
      ps.push_back(p);
    }
    run_igemm(ps);
    ps.clear();
    for (Group& g : groups) {
      if (j >= g.cfg->depth[0]) continue;
      ConvProblem p;
      linear(g, p, g.buf[7], g.cfg->block_aux_ch[0][j], pre + "ffn2.w", hd, pre + "ffn2.b", SNA_ACT_NONE, g.cur, g.buf[6]);
      ps.push_back(p);
    }
    run_igemm(ps);
    layernorm(pre + "ln2.g", pre + "ln2.b", j, 6, true);
  }
  // logits from token 0 of every request: a 1x1 "conv" over [n][S][1][hidden] with stride S
  conv_slot(a.n_classes % 8 != 0, [&](Group& g, ConvProblem& p) {
    p.x = g.cur; p.N = g.n; p.H = S; p.W = 1; p.C = hd;
    slice_conv(p, tensor("head.w"), a.n_classes, 1, S);
    p.Wo = 1; p.M = p.N * p.Ho * p.Wo;
    p.shift = (const float*)wptr(tensor("head.b"));
    p.y = logits_target(g, logits); p.out_fp32 = 1;
    return true;
  });
  scatter_logits(logits);
  if (hidden) {
    const size_t rb = (size_t)S * hd * T().esz;
    for (Group& g : groups) {
      std::vector<CopyItem> items;
      for (int i = 0; i < g.n; ++i) items.push_back({(size_t)i * rb, (size_t)g.reqs[i] * rb, rb});
      copy_items(g.cur, hidden, items);
    }
  }
  return SNA_OK;
}

// head of the workspace: the folded SubnetNorm tables, then the tile counters of reductions finished
// inside the matrix kernel (zeroed at load; every launch leaves them at zero)
static size_t folded_only_bytes(const ArchTables& T, int n_subnets) {
  return align_up((size_t)n_subnets * 2 * T.row_len * sizeof(float) + 256, 256);
}
static size_t folded_bytes(const ArchTables& T, int n_subnets) {
  return folded_only_bytes(T, n_subnets) + align_up(kTileCounters * sizeof(int), 256);
}
static size_t per_request_arena(const ArchTables& T) {
  return (size_t)NBUF * align_up(T.per_image_elems * T.esz, 256) + align_up(T.in_elems_max * T.esz, 256) +
         align_up(T.small_elems * 4, 256);
}

}  // namespace sna

using namespace sna;

// ---- recorded launch lists ---------------------------------------------------------------------
static hipError_t run_op(const PlanOp& op, hipStream_t s) {
  const char* a = op.args.data();
  switch (op.type) {
    case PlanOp::IGEMM: return launch_igemm(*(const ConvGroupArgs*)a, op.variant, op.flag != 0, s);
    case PlanOp::KREDUCE: return launch_splitk_reduce(*(const ConvGroupArgs*)a, s);
    case PlanOp::DIRECT: return launch_direct_conv(*(const ConvGroupArgs*)a, op.flag, s);
    case PlanOp::MAXPOOL: return launch_maxpool(*(const PoolGroupArgs*)a, op.flag, s);
    case PlanOp::GAP: return launch_gap(*(const PoolGroupArgs*)a, op.flag, s);
    case PlanOp::DW: return launch_depthwise(*(const DwGroupArgs*)a, s);
    case PlanOp::SE: return launch_se(*(const SeGroupArgs*)a, s);
    case PlanOp::LN: return launch_layernorm(*(const LnGroupArgs*)a, s);
    case PlanOp::ATTN: return launch_attention(*(const AttnGroupArgs*)a, s);
    case PlanOp::COPY: return launch_copy(*(const CopyArgs*)a, s);
    case PlanOp::PAD: return launch_pad_input(*(const PadArgs*)a, s);
    case PlanOp::STEMPOOL: return launch_stem_pool(*(const StemPoolArgs*)a, s);
    case PlanOp::MBV3HEAD: return launch_mbv3_head(*(const Mbv3HeadArgs*)a, s);
    case PlanOp::NORMCAL: return launch_norm_calibrate(*(const NormCalArgs*)a, s);
    case PlanOp::NORMAPPLY: return launch_norm_apply(*(const NormApplyArgs*)a, op.flag, s);
  }
  return hipErrorInvalidValue;
}

// Calls f(byte offset) for every pointer field of the op's arguments that may point at a caller
// buffer (activations in, results out; never weights or folded statistics).
template <class F>
static void visit_io_pointers(const PlanOp& op, F&& f) {
  const char* base = op.args.data();
  auto at = [&](const void* field) { f((int)((const char*)field - base)); };
  switch (op.type) {
    case PlanOp::IGEMM: case PlanOp::KREDUCE: case PlanOp::DIRECT: {
      const ConvGroupArgs* a = (const ConvGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].res); at(&a->p[i].y); }
      break;
    }
    case PlanOp::MAXPOOL: case PlanOp::GAP: {
      const PoolGroupArgs* a = (const PoolGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::DW: {
      const DwGroupArgs* a = (const DwGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::SE: {
      const SeGroupArgs* a = (const SeGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::LN: {
      const LnGroupArgs* a = (const LnGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::ATTN: {
      const AttnGroupArgs* a = (const AttnGroupArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].q); at(&a->p[i].k); at(&a->p[i].v); at(&a->p[i].o); }
      break;
    }
    case PlanOp::COPY: { const CopyArgs* a = (const CopyArgs*)base; at(&a->src); at(&a->dst); break; }
    case PlanOp::PAD: { const PadArgs* a = (const PadArgs*)base; at(&a->src); at(&a->dst); break; }
    case PlanOp::STEMPOOL: {
      const StemPoolArgs* a = (const StemPoolArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::MBV3HEAD: {
      const Mbv3HeadArgs* a = (const Mbv3HeadArgs*)base;
      for (int i = 0; i < a->n; ++i) { at(&a->p[i].x); at(&a->p[i].y); }
      break;
    }
    case PlanOp::NORMCAL: break;          // reads the scratch region, writes the statistics table
    case PlanOp::NORMAPPLY: { const NormApplyArgs* a = (const NormApplyArgs*)base; at(&a->res); at(&a->y); break; }
  }
}

// Run a launch list on the stream, with the per-launch event brackets when timing is enabled.
// Tuning key (M, K_out, C_in, taps, stride, parts, same-shaped problems in the launch) of the problem with the most work in a matrix-kernel
// launch: the one whose tile variant the whole launch uses.
static TuneKey lead_key(const PlanOp& op) {
  const ConvGroupArgs& a = *(const ConvGroupArgs*)op.args.data();
  int lead = 0;
  double lead_work = -1;
  for (int i = 0; i < a.n; ++i) {
    const ConvProblem& q = a.p[i];
    const double work = (double)q.M * q.K * (q.C * q.R * q.S + 64.0);
    if (work > lead_work) { lead_work = work; lead = i; }
  }
  const ConvProblem& q = a.p[lead];
  int twins = 0;
  for (int i = 0; i < a.n; ++i) {
    const ConvProblem& o = a.p[i];
    twins += o.M == q.M && o.K == q.K && o.C == q.C && o.R == q.R && o.S == q.S && o.stride == q.stride;
  }
  return {q.M, q.K, q.C, q.R * q.S, q.stride, q.parts, twins};
}

// One line of text for a launch: what the per-launch profile lists beside its time.
static std::string describe_op(const PlanOp& op) {
  char t[160];
  std::string out;
  if (op.type == PlanOp::IGEMM || op.type == PlanOp::KREDUCE || op.type == PlanOp::DIRECT) {
    const ConvGroupArgs& a = *(const ConvGroupArgs*)op.args.data();
    if (op.type == PlanOp::IGEMM) { snprintf(t, sizeof(t), "tile=%d chunked=%d", op.variant, op.flag); out = t; }
    for (int i = 0; i < a.n; ++i) {
      const ConvProblem& q = a.p[i];
      snprintf(t, sizeof(t), " [M=%d K=%d C=%d %dx%d/%d parts=%d tiles=%d]", q.M, q.K, q.C, q.R, q.S, q.stride, q.parts, q.tiles);
      out += t;
    }
  } else if (op.type == PlanOp::DW) {
    const DwGroupArgs& a = *(const DwGroupArgs*)op.args.data();
    for (int i = 0; i < a.n; ++i) {
      const DwProblem& q = a.p[i];
      snprintf(t, sizeof(t), " [N=%d H=%d C=%d %dx%d/%d]", q.N, q.H, q.C, q.k, q.k, q.stride);
      out += t;
    }
  } else if (op.type == PlanOp::SE) {
    const SeGroupArgs& a = *(const SeGroupArgs*)op.args.data();
    snprintf(t, sizeof(t), "phase=%d", op.flag); out = t;
    for (int i = 0; i < a.n; ++i) {
      snprintf(t, sizeof(t), " [N=%d HW=%d C=%d Q=%d]", a.p[i].N, a.p[i].HW, a.p[i].C, a.p[i].Q);
      out += t;
    }
  }
  return out;
}

static sna_status execute_plan(sna_supernet* net, const Plan& plan, hipStream_t stream) {
  for (const PlanOp& op : plan.ops) {
    hipEvent_t a = nullptr, b = nullptr;
    if (net->prof_on) {
      auto next_event = [&]() -> hipEvent_t {
        if (net->ev_used == net->ev_pool.size()) {
          hipEvent_t e;
          if (hipEventCreate(&e) != hipSuccess) return nullptr;
          net->ev_pool.push_back(e);
        }
        return net->ev_pool[net->ev_used++];
      };
      a = next_event(); b = next_event();
      if (a && b && hipEventRecord(a, stream) != hipSuccess) a = b = nullptr;
    }
    const hipError_t e = run_op(op, stream);
    if (e != hipSuccess) return fail(SNA_E_HIP, "launch failed: %s", hipGetErrorString(e));
    if (net->prof_on && a && b && hipEventRecord(b, stream) == hipSuccess) {
      ProfRec rec{op.kc, a, b, describe_op(op)};
      rec.flops = op.flops; rec.bytes = op.bytes;
      if (op.type == PlanOp::IGEMM) { rec.igemm = true; rec.key = lead_key(op); rec.variant = op.variant; }
      net->prof_recs.push_back(std::move(rec));
      net->prof_flops[op.kc] += op.flops;
      net->prof_bytes[op.kc] += op.bytes;
      net->prof_launches[op.kc] += 1;
    }
  }
  net->last_macs = plan.macs;
  net->last_launches = (int)plan.ops.size();
  return SNA_OK;
}

constexpr size_t kMaxPlans = 64;

// ---- static device scratch for the entry point that allocates nothing ---------------------------
// The per-call scratch of a forward (activation arena, input gather, small fp32 vectors, fp32 partial
// sums of split reductions) normally lives in the workspace the caller allocated.  Callers that cannot
// allocate get it from this array instead.  Each GPU holds its own copy at its own address, resolved
// once per device; host code only ever uses the resolved pointer.
constexpr size_t kStaticScratchBytes = (size_t)256 << 20;
constexpr size_t kStaticPartialBytes = (size_t)32 << 20;      // tail of the array: split-reduction partial sums
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (resolved on first use there), or nullptr with the
// error text set.
static char* static_scratch_base() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(SNA_E_HIP, "hipGetDevice: %s", e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fail(SNA_E_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = (char*)ptr;
  }
  return g_scratch_ptr[dev];
}

static sna_status forward_impl(sna_supernet* net, const sna_subnet_cfg* cfgs, int32_t n_cfgs, const int32_t* req_cfg,
                               int32_t n_requests, const void* inputs_dev, float* logits_dev, void* hidden_dev,
                               void* hip_stream, bool static_scratch);

extern "C" {

const char* sna_last_error(void) { return last_error_text(); }

int32_t sna_tensor_count(const sna_arch_desc* arch) {
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  return st != SNA_OK ? (int32_t)st : (int32_t)t.tensors.size();
}
int32_t sna_norm_count(const sna_arch_desc* arch) {
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  return st != SNA_OK ? (int32_t)st : (int32_t)t.norms.size();
}
sna_status sna_tensor_info_get(const sna_arch_desc* arch, int32_t index, sna_tensor_info* out) {
  if (!out) return fail(SNA_E_NULL, "out is NULL");
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  if (st != SNA_OK) return st;
  if (index < 0 || index >= (int)t.tensors.size()) return fail(SNA_E_ARCH, "tensor index %d", index);
  *out = t.tensors[index];
  return SNA_OK;
}
sna_status sna_norm_info_get(const sna_arch_desc* arch, int32_t index, sna_norm_info* out) {
  if (!out) return fail(SNA_E_NULL, "out is NULL");
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  if (st != SNA_OK) return st;
  if (index < 0 || index >= (int)t.norms.size()) return fail(SNA_E_ARCH, "norm index %d", index);
  *out = t.norms[index];
  return SNA_OK;
}
int64_t sna_weights_bytes(const sna_arch_desc* arch) {
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  return st != SNA_OK ? (int64_t)st : t.weight_bytes;
}
int64_t sna_stats_row_len(const sna_arch_desc* arch) {
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  return st != SNA_OK ? (int64_t)st : t.row_len;
}
int64_t sna_workspace_bytes(const sna_arch_desc* arch, int32_t n_subnets, int32_t max_batch) {
  ArchTables t;
  sna_status st = build_tables(arch, &t);
  if (st != SNA_OK) return (int64_t)st;
  if (n_subnets < 1 || max_batch < 1) return (int64_t)fail(SNA_E_BATCH, "n_subnets / max_batch < 1");
  return (int64_t)(folded_bytes(t, n_subnets) + (size_t)max_batch * per_request_arena(t) +
                   (size_t)SNA_MAX_GROUPS * 256 * (NBUF + 2) + kPartialBytes);
}

sna_status sna_supernet_load(const sna_arch_desc* arch, const void* weights_dev, size_t weights_bytes,
                             const void* stats_dev, size_t stats_bytes, int32_t n_subnets, int32_t max_batch,
                             void* workspace_dev, size_t workspace_bytes, void* hip_stream, sna_supernet** out) {
  if (!arch || !weights_dev || !workspace_dev || !out) return fail(SNA_E_NULL, "NULL argument");
  *out = nullptr;
  sna_supernet* net = new sna_supernet();
  sna_status st = build_tables(arch, &net->T);
  if (st != SNA_OK) { delete net; return st; }
  if (n_subnets < 1 || max_batch < 1) { delete net; return fail(SNA_E_BATCH, "n_subnets / max_batch < 1"); }
  if (net->T.row_len > 0 && !stats_dev) { delete net; return fail(SNA_E_NULL, "stats_dev is NULL"); }
  if (weights_bytes < (size_t)net->T.weight_bytes) {
    delete net;
    return fail(SNA_E_WORKSPACE, "weights blob %zu B < %lld B", weights_bytes, (long long)net->T.weight_bytes);
  }
  if (stats_bytes < (size_t)n_subnets * 4 * net->T.row_len * sizeof(float)) {
    delete net;
    return fail(SNA_E_WORKSPACE, "statistics table too small");
  }
  const int64_t need = sna_workspace_bytes(arch, n_subnets, max_batch);
  if ((int64_t)workspace_bytes < need) {
    delete net;
    return fail(SNA_E_WORKSPACE, "workspace %zu B < %lld B", workspace_bytes, (long long)need);
  }
  if (((uintptr_t)weights_dev | (uintptr_t)workspace_dev | (uintptr_t)stats_dev) & 255) {
    delete net;
    return fail(SNA_E_WORKSPACE, "buffers must be 256-byte aligned");
  }
  net->weights = (const char*)weights_dev;
  net->stats = (const float*)stats_dev;
  net->workspace = (char*)workspace_dev;
  net->workspace_bytes = workspace_bytes;
  net->folded = (float*)workspace_dev;
  net->arena = net->workspace + folded_bytes(net->T, n_subnets);
  net->arena_bytes = workspace_bytes - folded_bytes(net->T, n_subnets) - kPartialBytes;
  net->partials = net->arena + net->arena_bytes / 256 * 256;
  net->partials_bytes = kPartialBytes;
  net->counters = (int*)(net->workspace + folded_only_bytes(net->T, n_subnets));
  if (hipMemsetAsync(net->counters, 0, kTileCounters * sizeof(int), (hipStream_t)hip_stream) != hipSuccess) {
    delete net;
    return fail(SNA_E_HIP, "clearing the tile counters failed");
  }
  net->n_subnets = n_subnets;
  net->max_batch = max_batch;
  // resolve this device's static scratch now, outside any stream capture a later forward may run under
  // (a failure here is reported by the entry point that needs it)
  (void)static_scratch_base();
  hipError_t e = launch_fold_stats(net->stats, net->folded, n_subnets, net->T.row_len, (hipStream_t)hip_stream);
  if (e != hipSuccess) { delete net; return fail(SNA_E_HIP, "fold_stats: %s", hipGetErrorString(e)); }
  *out = net;
  return SNA_OK;
}

void sna_supernet_free(sna_supernet* net) {
  if (!net) return;
  for (hipEvent_t e : net->ev_pool) (void)hipEventDestroy(e);
  delete net;
}

sna_status sna_subnet_forward(sna_supernet* net, const sna_subnet_cfg* cfgs, int32_t n_cfgs,
                              const int32_t* req_cfg, int32_t n_requests, const void* inputs_dev,
                              float* logits_dev, void* hidden_dev, void* hip_stream) {
  return forward_impl(net, cfgs, n_cfgs, req_cfg, n_requests, inputs_dev, logits_dev, hidden_dev, hip_stream, false);
}

sna_status sna_subnet_forward_static(sna_supernet* net, const sna_subnet_cfg* cfgs, int32_t n_cfgs,
                                     const int32_t* req_cfg, int32_t n_requests, const void* inputs_dev,
                                     float* logits_dev, void* hidden_dev, void* hip_stream) {
  if (!net) return fail(SNA_E_NULL, "NULL argument");
  if (net->tuning || net->calibrating || net->prof_on)
    return fail(SNA_E_BATCH, "sna_subnet_forward_static: not while tuning, calibrating or profiling (those allocate)");
  return forward_impl(net, cfgs, n_cfgs, req_cfg, n_requests, inputs_dev, logits_dev, hidden_dev, hip_stream, true);
}

int64_t sna_static_scratch_bytes(void) { return (int64_t)kStaticScratchBytes; }

}  // extern "C"

// RAII: point the handle's per-call scratch at another region for the duration of one call
namespace {
struct ScratchSwap {
  sna_supernet* net;
  char *arena, *partials;
  size_t arena_bytes, partials_bytes;
  ScratchSwap(sna_supernet* n, char* base, size_t total, size_t part) : net(n), arena(n->arena), partials(n->partials),
      arena_bytes(n->arena_bytes), partials_bytes(n->partials_bytes) {
    n->arena = base; n->arena_bytes = total - part; n->partials = base + (total - part); n->partials_bytes = part;
  }
  ~ScratchSwap() { net->arena = arena; net->partials = partials; net->arena_bytes = arena_bytes; net->partials_bytes = partials_bytes; }
};
}  // namespace

static sna_status forward_impl(sna_supernet* net, const sna_subnet_cfg* cfgs, int32_t n_cfgs, const int32_t* req_cfg,
                               int32_t n_requests, const void* inputs_dev, float* logits_dev, void* hidden_dev,
                               void* hip_stream, bool static_scratch) {
  if (!net || !cfgs || !req_cfg) return fail(SNA_E_NULL, "NULL argument");
  if (n_requests < 0 || n_requests > net->max_batch)
    return fail(SNA_E_BATCH, "n_requests %d outside [0, %d]", n_requests, net->max_batch);
  if (n_cfgs < 1) return fail(SNA_E_BATCH, "n_cfgs < 1");
  if (n_requests == 0) { net->last_macs = 0; net->last_launches = 0; return SNA_OK; }
  if (!inputs_dev || !logits_dev) return fail(SNA_E_NULL, "NULL device buffer");
  if (((uintptr_t)inputs_dev | (uintptr_t)logits_dev) & 3) return fail(SNA_E_WORKSPACE, "inputs / logits must be 4-byte aligned");
  const ArchTables& T = net->T;
  const sna_arch_desc& a = T.arch;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (net->prof_on && net->prof_recs.size() > 200000) return fail(SNA_E_BATCH, "profile buffer full: call sna_profile_read");
  for (int r = 0; r < n_requests; ++r)
    if (req_cfg[r] < 0 || req_cfg[r] >= n_cfgs) return fail(SNA_E_BATCH, "req_cfg[%d]=%d outside [0, %d)", r, req_cfg[r], n_cfgs);

  std::unique_ptr<ScratchSwap> swap;
  if (static_scratch) {
    char* base = static_scratch_base();
    if (!base) return SNA_E_HIP;
    swap.reset(new ScratchSwap(net, base, kStaticScratchBytes, kStaticPartialBytes));
  }
  // The launch list depends on the routing, on the cfgs it names, on whether hidden states are
  // wanted, on where the scratch lives and on the tuning state; caller buffers only enter through
  // patched pointer fields.
  std::string key;
  const bool use_cache = net->plan_cache_on && !net->tuning && !net->calibrating;
  if (use_cache) {
    key.reserve((size_t)n_requests * 4 + 1024);
    const int32_t head[4] = {n_requests, hidden_dev ? 1 : 0, net->split_mode, static_scratch ? 1 : 0};
    key.append((const char*)head, sizeof(head));
    key.append((const char*)req_cfg, (size_t)n_requests * 4);
    std::vector<char> seen(n_cfgs, 0);
    for (int r = 0; r < n_requests; ++r)
      if (!seen[req_cfg[r]]) {
        seen[req_cfg[r]] = 1;
        key.append((const char*)&cfgs[req_cfg[r]], sizeof(sna_subnet_cfg));
      }
    for (Plan& pl : net->plans)
      if (pl.key == key) {
        const void* bases[3] = {inputs_dev, logits_dev, hidden_dev};
        for (const PlanPatch& pp : pl.patches)
          *(const char**)(pl.ops[pp.op].args.data() + pp.offset) = (const char*)bases[pp.which] + pp.delta;
        pl.last_use = ++net->plan_clock;
        return execute_plan(net, pl, stream);
      }
  }

  Fwd f;
  f.net = net;
  f.stream = stream;
  std::vector<int> gid(n_cfgs, -1);
  std::vector<size_t> req_off(n_requests), req_bytes(n_requests);
  size_t off = 0;
  for (int r = 0; r < n_requests; ++r) {
    const int ci = req_cfg[r];
    if (gid[ci] < 0) {
      sna_status st = validate_cfg(net, cfgs[ci]);
      if (st != SNA_OK) return st;
      if ((int)f.groups.size() == SNA_MAX_GROUPS) return fail(SNA_E_BATCH, "more than %d distinct cfgs in one call", SNA_MAX_GROUPS);
      gid[ci] = (int)f.groups.size();
      Group g;
      g.cfg = &cfgs[ci];
      g.cfg_index = ci;
      f.groups.push_back(g);
    }
    Group& g = f.groups[gid[ci]];
    if (g.n > 0 && g.reqs.back() != r - 1) g.contiguous = false;
    g.reqs.push_back(r);
    g.n++;
    const sna_subnet_cfg& c = cfgs[ci];
    const size_t elems = a.family == SNA_FAMILY_TRANSFORMER ? (size_t)c.in_h * a.hidden
                                                            : (size_t)c.in_h * c.in_w * a.in_ch;
    req_bytes[r] = elems * T.esz;
    req_off[r] = off;
    off += req_bytes[r];
  }
  // carve the arena: per group NBUF activation buffers, an input buffer and fp32 scratch
  char* cur = net->arena;
  const size_t act_b = align_up(T.per_image_elems * T.esz, 256);
  const size_t in_b = align_up(T.in_elems_max * T.esz, 256), sm_b = align_up(T.small_elems * 4, 256);
  for (Group& g : f.groups) {
    for (int i = 0; i < NBUF; ++i) { g.buf[i] = cur; cur += align_up(act_b * g.n, 256); }
    g.inbuf = cur; cur += align_up(in_b * g.n, 256);
    g.small = (float*)cur; cur += align_up(sm_b * g.n, 256);
  }
  if ((size_t)(cur - net->arena) > net->arena_bytes) {
    if (static_scratch)
      return fail(SNA_E_WORKSPACE, "these %d requests need %zu bytes of activation scratch; the static scratch holds %zu "
                  "(use sna_subnet_forward with a workspace, or a smaller batch)", n_requests, (size_t)(cur - net->arena),
                  net->arena_bytes);
    return fail(SNA_E_WORKSPACE, "arena overflow");
  }

  if (a.family == SNA_FAMILY_RESNET || a.family == SNA_FAMILY_MBV3)
    f.pad_inputs(inputs_dev, req_off, a.family == SNA_FAMILY_RESNET ? f.resnet_fused_stem() : f.mbv3_fused_head());
  else f.bind_inputs(inputs_dev, req_off, req_bytes);
  sna_status st;
  switch (a.family) {
    case SNA_FAMILY_TINY: st = f.run_tiny(inputs_dev, logits_dev); break;
    case SNA_FAMILY_RESNET: st = f.run_resnet(inputs_dev, logits_dev); break;
    case SNA_FAMILY_MBV3: st = f.run_mbv3(inputs_dev, logits_dev); break;
    case SNA_FAMILY_TRANSFORMER: st = f.run_transformer(inputs_dev, logits_dev, hidden_dev); break;
    default: st = fail(SNA_E_ARCH, "family");
  }
  if (st != SNA_OK) return st;
  if (f.err != hipSuccess) return fail(SNA_E_HIP, "launch failed: %s", hipGetErrorString(f.err));

  Plan plan;
  plan.ops = std::move(f.ops);
  plan.macs = f.macs;
  // pointer fields that landed inside a caller buffer get rewritten when the list is replayed
  const char* bases[3] = {(const char*)inputs_dev, (const char*)logits_dev, (const char*)hidden_dev};
  const size_t extents[3] = {off, (size_t)n_requests * a.n_classes * sizeof(float),
                             hidden_dev ? (size_t)n_requests * a.seq_len * a.hidden * T.esz : 0};
  for (size_t i = 0; i < plan.ops.size(); ++i)
    visit_io_pointers(plan.ops[i], [&](int offset) {
      const char* v = *(const char* const*)(plan.ops[i].args.data() + offset);
      for (int w = 0; w < 3; ++w)
        if (bases[w] && v >= bases[w] && v < bases[w] + extents[w]) {
          plan.patches.push_back({(int)i, offset, w, (size_t)(v - bases[w])});
          break;
        }
    });
  st = execute_plan(net, plan, stream);
  if (st == SNA_OK && use_cache) {
    plan.key = std::move(key);
    plan.last_use = ++net->plan_clock;
    if (net->plans.size() >= kMaxPlans) {                  // evict the least recently used list
      size_t lru = 0;
      for (size_t i = 1; i < net->plans.size(); ++i)
        if (net->plans[i].last_use < net->plans[lru].last_use) lru = i;
      net->plans[lru] = std::move(plan);
    } else {
      net->plans.push_back(std::move(plan));
    }
  }
  return st;
}

extern "C" {

sna_status sna_last_forward_info(const sna_supernet* net, int64_t* macs, int32_t* launches) {
  if (!net) return fail(SNA_E_NULL, "net is NULL");
  if (macs) *macs = net->last_macs;
  if (launches) *launches = net->last_launches;
  return SNA_OK;
}

static const char* kClassNames[SNA_N_KCLASS] = {"igemm_conv_linear", "direct_conv", "depthwise", "pool",
                                                "squeeze_excite", "layernorm", "attention", "copy",
                                                "fold_stats", "k_chunk_reduce", "stem_pool", "calibration"};
const char* sna_profile_class_name(int32_t k) { return (k >= 0 && k < SNA_N_KCLASS) ? kClassNames[k] : ""; }

sna_status sna_subnet_tune(sna_supernet* net, const sna_subnet_cfg* cfgs, int32_t n_cfgs, const int32_t* req_cfg,
                           int32_t n_requests, const void* inputs_dev, float* logits_dev, void* hidden_dev,
                           void* hip_stream) {
  if (!net) return fail(SNA_E_NULL, "net is NULL");
  std::set<TuneKey> known;
  for (const auto& kv : net->tuned) known.insert(kv.first);
  // Step 1: every new layer shape alone, launched back to back with each variant (also decides
  // whether a chunked reduction is split over blocks).
  net->tuning = true;
  net->plans.clear();                      // launch lists built before this call may use other tile variants
  sna_status st = sna_subnet_forward(net, cfgs, n_cfgs, req_cfg, n_requests, inputs_dev, logits_dev, hidden_dev, hip_stream);
  net->tuning = false;
  if (st == SNA_OK && hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return fail(SNA_E_HIP, "stream synchronize");
  bool any_new = false;
  for (const auto& kv : net->tuned) any_new = any_new || !known.count(kv.first);
  if (st != SNA_OK || !any_new || net->prof_on || n_requests == 0) return st;
  // Step 2: a layer launched back to back finds its operands in the caches, which it does not inside
  // a forward, and that changes which variant wins.  So the whole forward is run with every launch
  // forced to variant v, for each v in turn (rounds interleaved against clock drift), each launch
  // timed between two events; a new shape gets the variant with the least median time summed
  // over the launches it leads.
  const bool cache_was = net->plan_cache_on;
  const int forced_was = net->forced_variant;
  net->plan_cache_on = false;
  net->prof_on = true;
  const int nv = igemm_num_variants(), rounds = 7;
  std::map<TuneKey, std::vector<std::vector<double>>> samples;   // key -> [variant][round]
  for (int round = 0; round <= rounds && st == SNA_OK; ++round)             // round 0 warms up, not recorded
    for (int v = 0; v < nv && st == SNA_OK; ++v) {
      net->forced_variant = v;
      net->prof_recs.clear();
      net->ev_used = 0;
      st = sna_subnet_forward(net, cfgs, n_cfgs, req_cfg, n_requests, inputs_dev, logits_dev, hidden_dev, hip_stream);
      if (st != SNA_OK) break;
      std::map<TuneKey, double> sum;
      for (const ProfRec& r : net->prof_recs) {
        if (!r.igemm || r.variant != v) continue;       // a variant that cannot run this shape was not applied
        float ms = 0;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
        if (e != hipSuccess) { st = fail(SNA_E_HIP, "event: %s", hipGetErrorString(e)); break; }
        sum[r.key] += ms;
      }
      if (round == 0) continue;
      for (const auto& kv : sum) {
        auto& per_variant = samples[kv.first];
        per_variant.resize(nv);
        per_variant[v].push_back(kv.second);
      }
    }
  net->prof_recs.clear();
  net->ev_used = 0;
  for (int i = 0; i < SNA_N_KCLASS; ++i) { net->prof_launches[i] = 0; net->prof_flops[i] = 0; net->prof_bytes[i] = 0; }
  net->prof_on = false;
  net->plan_cache_on = cache_was;
  net->forced_variant = forced_was;
  if (st != SNA_OK) return st;
  for (auto& kv : samples) {
    if (known.count(kv.first)) continue;
    int best = -1;
    double best_t = 0;
    for (int v = 0; v < nv; ++v) {
      std::vector<double>& t = kv.second[v];
      if (t.empty()) continue;
      std::sort(t.begin(), t.end());
      const double med = t[t.size() / 2];
      if (best < 0 || med < best_t) { best = v; best_t = med; }
    }
    if (best >= 0) net->tuned[kv.first] = best;
  }
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return fail(SNA_E_HIP, "stream synchronize");
  // leave the caller's outputs as a plain forward would
  return sna_subnet_forward(net, cfgs, n_cfgs, req_cfg, n_requests, inputs_dev, logits_dev, hidden_dev, hip_stream);
}

sna_status sna_subnet_calibrate(sna_supernet* net, const sna_subnet_cfg* cfg, int32_t n_requests, const void* inputs_dev,
                                void* stats_dev, float* logits_dev, void* hip_stream) {
  if (!net || !cfg || !inputs_dev || !stats_dev || !logits_dev) return fail(SNA_E_NULL, "NULL argument");
  if (net->T.row_len == 0) return fail(SNA_E_ARCH, "this architecture has no SubnetNorm layers");
  if ((const float*)stats_dev != net->stats) return fail(SNA_E_BATCH, "stats_dev is not the table this SuperNet was loaded with");
  if (n_requests < 1) return fail(SNA_E_BATCH, "calibration needs at least one request");
  std::vector<int32_t> route((size_t)n_requests, 0);
  const int split_was = net->split_mode;
  net->calibrating = true;
  net->stats_mut = (float*)stats_dev;
  net->split_mode = 1;                       // the fp32 scratch region holds the layers' raw outputs
  sna_status st = sna_subnet_forward(net, cfg, 1, route.data(), n_requests, inputs_dev, logits_dev, nullptr, hip_stream);
  net->calibrating = false;
  net->stats_mut = nullptr;
  net->split_mode = split_was;
  if (st == SNA_E_HIP && strstr(sna_last_error(), "out of memory"))
    return fail(SNA_E_WORKSPACE, "calibration batch too large: a layer's fp32 output does not fit the %zu MiB scratch region",
                kPartialBytes >> 20);
  return st;
}

int32_t sna_tuned_count(const sna_supernet* net) { return net ? (int32_t)(net->tuned.size() + net->tuned_split.size()) : 0; }

int64_t sna_tuning_export(const sna_supernet* net, char* buf, int64_t cap) {
  if (!net) return (int64_t)fail(SNA_E_NULL, "net is NULL");
  std::string out;
  char line[128];
  for (const auto& kv : net->tuned) {
    snprintf(line, sizeof(line), "v %d %d %d %d %d %d %d %d\n", kv.first[0], kv.first[1], kv.first[2], kv.first[3],
             kv.first[4], kv.first[5], kv.first[6], kv.second);
    out += line;
  }
  for (const auto& kv : net->tuned_split) {
    snprintf(line, sizeof(line), "s %d %d %d %d %d %d %d %d\n", kv.first[0], kv.first[1], kv.first[2], kv.first[3],
             kv.first[4], kv.first[5], kv.first[6], kv.second);
    out += line;
  }
  if (buf && cap > 0) {
    const size_t ncopy = std::min<size_t>(out.size(), (size_t)cap);
    memcpy(buf, out.data(), ncopy);
    if ((int64_t)out.size() < cap) buf[out.size()] = 0;
  }
  return (int64_t)out.size();
}

sna_status sna_tuning_import(sna_supernet* net, const char* text, int64_t len) {
  if (!net || !text) return fail(SNA_E_NULL, "NULL argument");
  std::map<TuneKey, int> tv, ts;
  const std::string all(text, (size_t)(len < 0 ? 0 : len));
  size_t pos = 0;
  while (pos < all.size()) {
    size_t end = all.find('\n', pos);
    if (end == std::string::npos) end = all.size();
    const std::string ln = all.substr(pos, end - pos);
    pos = end + 1;
    if (ln.empty() || ln[0] == '#') continue;
    char kind = 0, extra = 0;
    int k[7], val = 0;
    // key of seven numbers and the choice; a line with six (written before the twin count existed) means one twin
    const int got = sscanf(ln.c_str(), "%c %d %d %d %d %d %d %d %d %c", &kind, &k[0], &k[1], &k[2], &k[3], &k[4], &k[5], &k[6], &val, &extra);
    if (got == 8) { val = k[6]; k[6] = 1; }
    else if (got != 9) return fail(SNA_E_CFG_RANGE, "tuning line not understood: %s", ln.c_str());
    if (k[6] < 1) return fail(SNA_E_CFG_RANGE, "tuning line out of range: %s", ln.c_str());
    const TuneKey key = {k[0], k[1], k[2], k[3], k[4], k[5], k[6]};
    if (kind == 'v' && val >= 0 && val < igemm_num_variants()) tv[key] = val;
    else if (kind == 's' && (val == 0 || val == 1)) ts[key] = val;
    else return fail(SNA_E_CFG_RANGE, "tuning line out of range: %s", ln.c_str());
  }
  for (const auto& kv : tv) net->tuned[kv.first] = kv.second;
  for (const auto& kv : ts) net->tuned_split[kv.first] = kv.second;
  net->plans.clear();
  return SNA_OK;
}

int32_t sna_tile_variant_count(void) { return igemm_num_variants(); }

sna_status sna_set_tile_variant(sna_supernet* net, int32_t variant) {
  if (!net) return fail(SNA_E_NULL, "net is NULL");
  if (variant < -1 || variant >= igemm_num_variants()) return fail(SNA_E_CFG_RANGE, "tile variant %d", variant);
  net->forced_variant = variant;
  net->plans.clear();
  return SNA_OK;
}

sna_status sna_set_k_split(sna_supernet* net, int32_t mode) {
  if (!net) return fail(SNA_E_NULL, "net is NULL");
  if (mode < 0 || mode > 3) return fail(SNA_E_CFG_RANGE, "k split mode %d", mode);
  net->split_mode = mode;
  net->plans.clear();
  return SNA_OK;
}

sna_status sna_profile_enable(sna_supernet* net, int32_t on) {
  if (!net) return fail(SNA_E_NULL, "net is NULL");
  net->prof_on = on != 0;
  return SNA_OK;
}

int64_t sna_profile_read_launches(sna_supernet* net, char* buf, int64_t cap) {
  if (!net) { fail(SNA_E_NULL, "net is NULL"); return -1; }
  std::string out;
  char t[160];
  for (const ProfRec& r : net->prof_recs) {
    hipError_t e = hipEventSynchronize(r.b);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) { fail(SNA_E_HIP, "event: %s", hipGetErrorString(e)); return -1; }
    snprintf(t, sizeof(t), "%.3f %s flops=%.0f bytes=%.0f ", ms * 1e3, kClassNames[r.kc], r.flops, r.bytes);
    out += t; out += r.what; out += '\n';
  }
  if (buf && cap > 0) {
    const size_t ncopy = std::min((size_t)cap - 1, out.size());
    memcpy(buf, out.data(), ncopy);
    buf[ncopy] = 0;
  }
  return (int64_t)out.size();
}

sna_status sna_profile_read(sna_supernet* net, double ms[SNA_N_KCLASS], int64_t launches[SNA_N_KCLASS],
                            double flops[SNA_N_KCLASS], double bytes[SNA_N_KCLASS]) {
  if (!net || !ms || !launches || !flops || !bytes) return fail(SNA_E_NULL, "NULL argument");
  for (int i = 0; i < SNA_N_KCLASS; ++i) ms[i] = 0;
  for (const ProfRec& r : net->prof_recs) {
    hipError_t e = hipEventSynchronize(r.b);
    float t = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
    if (e != hipSuccess) return fail(SNA_E_HIP, "event: %s", hipGetErrorString(e));
    ms[r.kc] += t;
  }
  for (int i = 0; i < SNA_N_KCLASS; ++i) {
    launches[i] = net->prof_launches[i]; flops[i] = net->prof_flops[i]; bytes[i] = net->prof_bytes[i];
    net->prof_launches[i] = 0; net->prof_flops[i] = 0; net->prof_bytes[i] = 0;
  }
  net->prof_recs.clear();
  net->ev_used = 0;
  return SNA_OK;
}

}  // extern "C"
