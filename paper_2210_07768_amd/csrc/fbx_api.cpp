// C ABI of libfbx: plan lifetime, workspace layout, and the launch sequence of
// one extraction call.  See include/fbx.h for the contract of every entry point.
#include <algorithm>
#include <cmath>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "fbx_device.h"

using namespace fbx;

namespace {

constexpr uint64_t kAlign = 256;
uint64_t align_up(uint64_t x, uint64_t a = kAlign) { return (x + a - 1) / a * a; }

thread_local std::string g_create_error;

struct Timer {
  hipEvent_t ev[2] = {nullptr, nullptr};
  bool used = false;
};

}  // namespace

struct fbx_plan {
  PlanHost host;
  std::string error;

  // workspace
  uint8_t* ws = nullptr;
  uint64_t ws_bytes = 0;
  // constant-table placement inside the workspace (byte offsets)
  uint64_t off_ctrl = 0, off_dyn = 0, off_ops = 0, off_layer_ops = 0, off_layer_begin = 0, off_nonroot = 0,
           off_aux = 0, off_fields = 0, off_field_ops = 0, off_prog_ops = 0, off_prog_fields = 0, off_row_total = 0,
           off_tile_lists = 0, off_tile_list_begin = 0, off_rnr = 0, off_prof = 0, off_actual = 0, off_cap = 0, off_static_end = 0;

  // options
  int fused = 1;
  int tile_engine = 1;            // 0: the walk kernels also when all layers share a launch
  uint32_t lds_pad = 0;
  int profile = 0;
  int tile_log2 = -1;             // -1: chosen per call
  uint32_t raw_cap = 0;           // 0: chosen per call
  uint32_t lds_budget = 80u * 1024u;  // two workgroups per compute unit
  uint32_t dbg = 0;
  uint32_t grid_limit = 0;
  uint32_t spin_limit = 1u << 22;   // polls a tile of the one-launch sequence waits for an earlier tile's count
  int one_launch = 1;             // size ragged arrays from the last call and skip the counting launch
  uint32_t passes_skip = 0, passes_backoff = 0;  // calls that do not try the one-launch sequence after a tile did not fit its LDS section; how many next time
  int placement = 0;              // one-launch sequence: 0 tiles placed in record order (look-back), 1 in the order they arrive (one atomic add each)
  int compile = 0;                // compile the tile kernel for this plan at run time (Section 4's meta-kernel)
  uint32_t tile_threads = 512;    // lanes of a workgroup of the kernels compiled for the plan
  uint32_t lane_ops = 0;          // tiles of 64 records in compiled kernels: how single-sign operators run (see fbx_tile.hip)
  TileJit jit;

  // what the last successful call taught about ragged sizes (signs per ragged operator)
  bool learned = false;
  uint64_t learned_records = 0;
  std::vector<uint64_t> learned_total;   // by ragged row
  std::vector<uint64_t> cap_host;        // capacities of the current call, by ragged row
  int last_mode = 0;                     // 1: counting + writing launch, 2: one launch
  uint64_t margin_failed_ws = 0;         // workspace size at which the sized arrays did not fit (no retry below it)

  uint64_t id = 0;                // unique among the plans of this process (a destroyed plan's address may come back)
  std::vector<uint8_t> tables;    // image of the constant tables, as they lie at the head of a workspace

  // results of the last call
  std::vector<uint8_t> readback;  // Ctrl + OpDyn[n_ops]
  std::vector<fbx_slot_view> slots;
  std::vector<uint32_t> emitted;  // operator index of every emitted slot, spec order

  // profiling
  std::vector<Timer> timers;  // 0 validate, 1 count, 2 scan, 3 alloc, 4.. tile launches
  uint32_t n_tile_launches = 0;
  std::vector<uint32_t> tile_launch_layer;

  void layout() {
    const uint64_t n = host.ops.size();
    uint64_t o = 0;
    off_ctrl = o; o += sizeof(Ctrl);
    off_dyn = o; o += n * sizeof(OpDyn);
    off_actual = o; o = align_up(o + host.n_ragged * 8ull);  // read back together with the placements
    off_ops = o; o = align_up(o + n * sizeof(OpDesc));
    off_layer_ops = o; o = align_up(o + n * 4);
    off_layer_begin = o; o = align_up(o + (host.n_layers + 1) * 4);
    off_nonroot = o; o = align_up(o + host.nonroot_ops.size() * 4);
    off_aux = o; o = align_up(o + host.aux.size());
    off_fields = o; o = align_up(o + host.fields.size() * sizeof(FieldDesc));
    off_field_ops = o; o = align_up(o + host.field_ops.size() * 4);
    off_prog_ops = o; o = align_up(o + n * sizeof(OpProg));
    off_prog_fields = o; o = align_up(o + host.fields.size() * sizeof(FieldProg));
    off_row_total = o; o = align_up(o + host.n_ragged * 8ull);
    off_tile_lists = o; o = align_up(o + host.tile_lists.size() * 4);
    off_tile_list_begin = o; o = align_up(o + host.tile_list_begin.size() * 4);
    off_rnr = o; o = align_up(o + host.derive_tab.size() * 4);
    off_prof = o; o = align_up(o + 32 * 8);
    off_cap = o; o = align_up(o + host.n_ragged * 8ull);
    off_static_end = o;
  }

  void build_tables() {
    const PlanHost& h = host;
    tables.assign(off_static_end, 0);
    uint8_t* img = tables.data();
    std::vector<OpDesc> descs(h.ops.size());
    for (size_t i = 0; i < h.ops.size(); ++i) descs[i] = h.ops[i].d;
    if (!descs.empty()) std::memcpy(img + off_ops, descs.data(), descs.size() * sizeof(OpDesc));
    if (!h.layer_ops.empty()) std::memcpy(img + off_layer_ops, h.layer_ops.data(), h.layer_ops.size() * 4);
    std::memcpy(img + off_layer_begin, h.layer_begin.data(), h.layer_begin.size() * 4);
    if (!h.nonroot_ops.empty()) std::memcpy(img + off_nonroot, h.nonroot_ops.data(), h.nonroot_ops.size() * 4);
    if (!h.aux.empty()) std::memcpy(img + off_aux, h.aux.data(), h.aux.size());
    if (!h.fields.empty()) std::memcpy(img + off_fields, h.fields.data(), h.fields.size() * sizeof(FieldDesc));
    if (!h.field_ops.empty()) std::memcpy(img + off_field_ops, h.field_ops.data(), h.field_ops.size() * 4);
    if (!h.tile_lists.empty()) std::memcpy(img + off_tile_lists, h.tile_lists.data(), h.tile_lists.size() * 4);
    std::memcpy(img + off_tile_list_begin, h.tile_list_begin.data(), h.tile_list_begin.size() * 4);
    if (!h.derive_tab.empty()) std::memcpy(img + off_rnr, h.derive_tab.data(), h.derive_tab.size() * 4);
  }
};

namespace {

struct CallGeometry {
  bool tile_engine = false;
  uint32_t n_tiles = 0, count_waves = 1;
  uint64_t off_tile_cnt = 0, off_tile_base = 0, off_scan_part = 0, arena_base = 0;
  TileParams tp{};  // LDS layout and tile size (tile engine only)
};

uint32_t round16(uint64_t x) { return static_cast<uint32_t>((x + 15u) & ~uint64_t(15)); }

// LDS layout of the tile kernel for tiles of 2^lt records and raw_cap staged bytes.
void tile_lds_layout(const PlanHost& h, uint32_t lt, uint32_t raw_cap, TileParams& tp) {
  const uint32_t T = 1u << lt;
  tp.n_mh = tp.n_split = 0;  // (the list is sorted: multi-valued hashes, other multi-valued operators, the rest)
  for (uint32_t i = h.tile_list_begin[TL_RAGROOT]; i < h.tile_list_begin[TL_RAGROOT + 1]; ++i) {
    const OpDesc& d = h.ops[h.tile_lists[i]].d;
    if (d.kind == OP_HASH) ++tp.n_mh;
    if (d.flags & F_MULTI) ++tp.n_split;
  }
  tp.log2T = lt;
  tp.raw_cap = raw_cap;
  tp.row_stride = (h.n_fields + 1u) | 1u;  // odd: neighbouring records start in different banks
  uint32_t o = 0;
  tp.o_off = o; o = round16(o + 2 * 8ull * (T + 1));  // this tile's offsets and the next one's
  tp.o_rs = o; o = round16(o + 4ull * T);
  tp.o_re = o; o = round16(o + 4ull * T);
  tp.o_rows = o; o = round16(o + 2ull * T * tp.row_stride);
  tp.o_raw = o; o = round16(o + kRawPad + uint64_t(raw_cap) + 32u);
  tp.o_stage = o; o = round16(o + 8ull * T * h.n_stage);
  tp.o_cnt = o; o = round16(o + 4ull * T * h.n_ragged);
  tp.o_start = o; o = round16(o + 4ull * T * h.n_ragged);
  tp.o_run = o; o = round16(o + 4ull * h.n_ragged);
  tp.o_base = o; o = round16(o + 8ull * h.n_ragged);
  tp.o_tot = o; o = round16(o + 4ull * h.n_ragged);
  tp.o_cap = o; o = round16(o + 8ull * h.n_ragged);
  tp.n_gen = 0;
  for (uint32_t layer = 2; layer <= h.n_layers; ++layer) {
    const uint32_t list = TL_LAYER + 2u * (layer - 2u) + 1u;
    tp.n_gen += h.tile_list_begin[list + 1] - h.tile_list_begin[list];
  }
  tp.o_gfirst = o; o = round16(o + (tp.n_gen ? 4ull * h.ops.size() : 0ull));
  tp.o_gtot = o; o = round16(o + (tp.n_gen ? 4ull * (h.n_layers + 1u) : 0ull));
  tp.o_ioff = o; o = round16(o + 4ull * (tp.n_mh + 1));
  tp.item_cap = 16;
  tp.o_ctab = o; o = round16(o + 2ull * tp.n_mh * T * tp.item_cap);
  tp.o_prog = o; o = round16(o + sizeof(OpProg) * h.ops.size());
  tp.o_lbeg = o; o = round16(o + 4ull * h.tile_list_begin.size());
  tp.o_rnr = o; o = round16(o + 4ull * h.derive_tab.size());
  tp.o_aux = o; o = round16(o + h.aux.size());
  tp.lds_bytes = o;
}

// Tile size: the largest power of two (at most 64 records) whose LDS sections
// stay inside the budget when the staged text is sized for 1.25 times the mean
// record length.  Returns false when even one record per tile does not fit the
// device (very wide plans): the walk kernels then take the call.
bool tile_geometry(const fbx_plan& p, uint64_t raw_len, uint64_t n_records, TileParams& tp) {
  const PlanHost& h = p.host;
  if (h.n_fields > 32000 || h.ops.size() > 2048 || h.aux.size() > 65536) return false;
  const uint64_t avg = n_records ? (raw_len + n_records - 1) / n_records : 0;
  const uint32_t dev_max = tile_max_lds();
  const int lt_hi = p.tile_log2 >= 0 ? p.tile_log2 : 6, lt_lo = p.tile_log2 >= 0 ? p.tile_log2 : 0;
  for (int lt = lt_hi; lt >= lt_lo; --lt) {
    uint64_t want = (uint64_t(1) << lt) * avg * 5 / 4 + 64;
    if (p.compile) {
      // kernels compiled for the plan are compiled for one section size: batches of about the
      // same record length must agree on it, so sizes go up in steps of an eighth of a power of two
      uint64_t step = 128;
      while (step * 16 <= want) step <<= 1;
      want = (want + step - 1) / step * step;
    }
    const uint32_t cap = p.raw_cap ? p.raw_cap : round16(std::min<uint64_t>(std::max<uint64_t>(want, 1024), 65000));
    tile_lds_layout(h, static_cast<uint32_t>(lt), cap, tp);
    const uint32_t limit = (lt == lt_lo) ? dev_max : std::min(p.lds_budget, dev_max);
    if (tp.lds_bytes <= limit) return true;
  }
  return false;
}

CallGeometry geometry(const fbx_plan& p, uint64_t raw_len, uint64_t n_records) {
  CallGeometry g;
  g.tile_engine = p.fused && p.tile_engine && tile_geometry(p, raw_len, n_records, g.tp);
  if (g.tile_engine) {
    g.n_tiles = static_cast<uint32_t>((n_records + (1ull << g.tp.log2T) - 1) >> g.tp.log2T);
  } else {
    g.n_tiles = static_cast<uint32_t>((n_records + kTile - 1) >> kTileLog2);
    // counting pass: one 256-byte LDS row per ragged operator and wavefront; as many
    // wavefronts per workgroup (at most 4) as fit into 48 KB
    const uint32_t per_wave = 8960u + p.host.n_ragged * 256u;  // byte ring + count rows
    g.count_waves = std::min(4u, std::max(1u, 65536u / per_wave));
  }
  uint64_t w = p.off_static_end;
  g.off_tile_cnt = w; w = align_up(w + uint64_t(p.host.n_ragged) * g.n_tiles * 4);
  g.off_tile_base = w; w = align_up(w + uint64_t(p.host.n_ragged) * g.n_tiles * 8);
  g.off_scan_part = w; w = align_up(w + uint64_t(p.host.n_ragged) * scan_segments(g.n_tiles) * 8);
  g.arena_base = w;
  return g;
}

fbx_status hip_fail(fbx_plan* p, hipError_t e, const char* where) {
  p->error = std::string(where) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();
  return FBX_E_HIP;
}

}  // namespace

extern "C" {

const char* fbx_status_str(fbx_status s) {
  switch (s) {
    case FBX_OK: return "ok";
    case FBX_E_ARG: return "bad argument";
    case FBX_E_SPEC: return "bad operator spec";
    case FBX_E_NOMEM: return "workspace too small";
    case FBX_E_INPUT: return "bad record offsets";
    case FBX_E_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* fbx_last_error(const fbx_plan* plan) { return plan ? plan->error.c_str() : g_create_error.c_str(); }

fbx_status fbx_plan_create(const char* spec, size_t spec_len, fbx_plan** out) {
  if (!spec || !out) {
    g_create_error = "spec and out must not be NULL";
    return FBX_E_ARG;
  }
  std::unique_ptr<fbx_plan> p(new (std::nothrow) fbx_plan());
  if (!p) return FBX_E_ARG;
  std::string err;
  fbx_status st = parse_plan(spec, spec_len, p->host, err);
  if (st != FBX_OK) {
    g_create_error = err;
    return st;
  }
  for (uint32_t i = 0; i < p->host.ops.size(); ++i)
    if (p->host.ops[i].d.flags & F_EMIT) p->emitted.push_back(i);
  p->slots.resize(p->emitted.size());
  p->layout();
  p->readback.resize(p->off_actual + p->host.n_ragged * 8ull);
  p->build_tables();
  static std::atomic<uint64_t> next_id{1};
  p->id = next_id.fetch_add(1);
  *out = p.release();
  return FBX_OK;
}

void fbx_plan_destroy(fbx_plan* plan) {
  if (!plan) return;
  for (Timer& t : plan->timers)
    for (hipEvent_t e : t.ev)
      if (e) (void)hipEventDestroy(e);
  delete plan;
}

fbx_status fbx_plan_compiled(const fbx_plan* plan, uint32_t* n_kernels, double* ms) {
  if (!plan) return FBX_E_ARG;
  if (n_kernels) *n_kernels = plan->jit.compiled();
  if (ms) *ms = plan->jit.compile_ms();
  return FBX_OK;
}

fbx_status fbx_plan_kernel_source(const fbx_plan* plan, uint64_t raw_len, uint64_t n_records, int mode, char* buf,
                                  size_t buf_len, size_t* needed) {
  if (!plan || mode < 0 || mode > 3 || (!buf && buf_len)) return FBX_E_ARG;
  const CallGeometry g = geometry(*plan, raw_len, n_records);
  if (!g.tile_engine) return FBX_E_ARG;  // (plans too wide for the tile kernel have no such kernel)
  TileParams Q = g.tp;
  const PlanHost& h = plan->host;
  Q.n_ops = static_cast<uint32_t>(h.ops.size()); Q.n_layers = h.n_layers; Q.n_ragged = h.n_ragged;
  Q.n_rnr = h.n_derive;
  Q.rnr_words = static_cast<uint32_t>(h.derive_tab.size());
  Q.alias_at = h.alias_at; Q.n_alias = h.n_alias;
  Q.n_lists = static_cast<uint32_t>(h.tile_list_begin.size()) - 1u;
  Q.aux_bytes = static_cast<uint32_t>(h.aux.size());
  Q.n_fields = h.n_fields; Q.n_stage = h.n_stage;
  Q.lds_bytes = std::max(Q.lds_bytes, plan->lds_pad);
  const std::string text = tile_kernel_source(Q, mode, h, plan->tile_threads, plan->lane_ops);
  if (needed) *needed = text.size() + 1;
  if (buf_len) {
    const size_t n = std::min(buf_len - 1, text.size());
    std::memcpy(buf, text.data(), n);
    buf[n] = 0;
  }
  return FBX_OK;
}

fbx_status fbx_plan_info(const fbx_plan* plan, uint32_t* n_ops, uint32_t* n_layers, uint32_t* layer_of_op,
                         uint32_t* arity_of_op) {
  if (!plan) return FBX_E_ARG;
  if (n_ops) *n_ops = static_cast<uint32_t>(plan->host.ops.size());
  if (n_layers) *n_layers = plan->host.n_layers;
  for (size_t i = 0; i < plan->host.ops.size(); ++i) {
    if (layer_of_op) layer_of_op[i] = plan->host.ops[i].d.layer;
    if (arity_of_op) arity_of_op[i] = plan->host.ops[i].d.arity;
  }
  return FBX_OK;
}

fbx_status fbx_plan_set_option(fbx_plan* plan, const char* key, int64_t value) {
  if (!plan || !key) return FBX_E_ARG;
  const std::string k(key);
  if (k == "fused") {
    if (value != 0 && value != 1) { plan->error = "fused must be 0 or 1"; return FBX_E_ARG; }
    plan->fused = static_cast<int>(value);
  } else if (k == "tile_engine") {
    if (value != 0 && value != 1) { plan->error = "tile_engine must be 0 or 1"; return FBX_E_ARG; }
    plan->tile_engine = static_cast<int>(value);
  } else if (k == "lds_pad") {
    if (value < 0 || value > 65536) { plan->error = "lds_pad must be in 0..65536"; return FBX_E_ARG; }
    plan->lds_pad = static_cast<uint32_t>(value);
  } else if (k == "tile_log2") {
    if (value < -1 || value > 6) { plan->error = "tile_log2 must be in -1..6"; return FBX_E_ARG; }
    plan->tile_log2 = static_cast<int>(value);
  } else if (k == "raw_cap") {
    if (value < 0 || value > 65000 || (value && value < 64)) { plan->error = "raw_cap must be 0 or in 64..65000"; return FBX_E_ARG; }
    plan->raw_cap = static_cast<uint32_t>(value) & ~15u;
  } else if (k == "lds_budget") {
    if (value < 4096 || value > 160 * 1024) { plan->error = "lds_budget must be in 4096..163840"; return FBX_E_ARG; }
    plan->lds_budget = static_cast<uint32_t>(value);
  } else if (k == "compile") {
    if (value != 0 && value != 1) { plan->error = "compile must be 0 or 1"; return FBX_E_ARG; }
    plan->compile = static_cast<int>(value);
  } else if (k == "lane_ops") {
    if (value < 0 || value > 2) { plan->error = "lane_ops must be 0, 1 or 2"; return FBX_E_ARG; }
    plan->lane_ops = static_cast<uint32_t>(value);
  } else if (k == "tile_threads") {
    if (value != 512 && value != 1024) { plan->error = "tile_threads must be 512 or 1024"; return FBX_E_ARG; }
    plan->tile_threads = static_cast<uint32_t>(value);
  } else if (k == "placement") {
    if (value != 0 && value != 1) { plan->error = "placement must be 0 (record order) or 1 (arrival order)"; return FBX_E_ARG; }
    plan->placement = static_cast<int>(value);
  } else if (k == "one_launch") {
    if (value != 0 && value != 1) { plan->error = "one_launch must be 0 or 1"; return FBX_E_ARG; }
    plan->one_launch = static_cast<int>(value);
  } else if (k == "spin_limit") {
    if (value < 0 || value > (1ll << 30)) { plan->error = "spin_limit must be in 0..2^30"; return FBX_E_ARG; }
    plan->spin_limit = static_cast<uint32_t>(value);
  } else if (k == "grid_limit") {
    if (value < 0 || value > 65536) { plan->error = "grid_limit must be in 0..65536"; return FBX_E_ARG; }
    plan->grid_limit = static_cast<uint32_t>(value);
#ifdef FBX_TILE_PROF
  } else if (k == "debug_skip") {  // tuning builds: leave phases out (results are then wrong)
    plan->dbg = static_cast<uint32_t>(value);
#endif
  } else if (k == "profile") {
    if (value != 0 && value != 1) { plan->error = "profile must be 0 or 1"; return FBX_E_ARG; }
    plan->profile = static_cast<int>(value);
  } else {
    plan->error = "unknown option '" + k + "'";
    return FBX_E_ARG;
  }
  return FBX_OK;
}

fbx_status fbx_plan_workspace_hint(const fbx_plan* plan, uint64_t raw_len, uint64_t n_records, uint64_t* bytes) {
  if (!plan || !bytes) return FBX_E_ARG;
  const CallGeometry g = geometry(*plan, raw_len, n_records);
  // fixed-arity operators are exact; a ragged root operator cannot emit more
  // signs than its field has bytes + 1, for which raw_len / #fields + records
  // is a fair guess; a ragged cross or concat is guessed at four times that.
  const uint64_t per_root = raw_len / std::max(plan->host.n_fields, 1u) + n_records;
  uint64_t total = g.arena_base;
  for (const HostOp& op : plan->host.ops) {
    uint64_t n = op.d.arity ? n_records * op.d.arity : (op.d.layer == 1 ? per_root : 4 * per_root);
    total += align_up(n * 8, 128);
    if (!op.d.arity) total += align_up((n_records + 1) * 8, 128);
  }
  *bytes = align_up(total + 4096);
  return FBX_OK;
}

fbx_status fbx_plan_set_workspace(fbx_plan* plan, void* d_workspace, uint64_t bytes) {
  if (!plan || !d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255u)) {
    if (plan) plan->error = "workspace must be a non-NULL, 256-byte aligned device pointer";
    return FBX_E_ARG;
  }
  if (bytes < plan->off_static_end) {
    plan->error = "workspace smaller than the plan's constant tables (" + std::to_string(plan->off_static_end) + " bytes)";
    return FBX_E_NOMEM;
  }
  hipError_t e = hipMemcpy(d_workspace, plan->tables.data(), plan->tables.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) return hip_fail(plan, e, "copying plan tables");
  plan->ws = static_cast<uint8_t*>(d_workspace);
  plan->ws_bytes = bytes;
  return FBX_OK;
}

}  // extern "C"

namespace {

// Where one call keeps its memory.  With a workspace everything lies in it: the tables first,
// the arena (the operators' arrays) from arena_base on.  The entry point that allocates nothing
// keeps the tables in the library's own device array and the arena in the caller's output buffer.
struct Regions {
  uint8_t* tables;       // control block, plan tables, per-call and per-tile tables
  uint64_t tables_cap;   // bytes there
  uint64_t origin;       // address that array offsets count from (arena byte 0 lies at origin + arena_base)
  uint64_t cap;          // array offsets must stay below this
  bool own_tables;       // the tables are the library's array: no run-time compilation, no event creation
};

fbx_status extract_impl(fbx_plan* plan, const uint8_t* d_raw, uint64_t raw_len, const uint64_t* d_rec_off,
                        uint64_t n_records, void* hip_stream, fbx_result* out, const Regions& reg, const CallGeometry& g) {
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const PlanHost& h = plan->host;
  const uint32_t n_ops = static_cast<uint32_t>(h.ops.size());
  uint8_t* ws = reg.tables;
  const uint64_t ws_bytes = reg.cap;
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + plan->off_ctrl);
  OpDyn* dyn = reinterpret_cast<OpDyn*>(ws + plan->off_dyn);
  WalkParams P{};
  P.raw = d_raw; P.raw_len = raw_len; P.rec_off = d_rec_off; P.n_records = n_records;
  P.origin = reg.origin;
  P.ops = reinterpret_cast<const OpDesc*>(ws + plan->off_ops);
  P.fields = reinterpret_cast<const FieldDesc*>(ws + plan->off_fields);
  P.field_ops = reinterpret_cast<const uint32_t*>(ws + plan->off_field_ops);
  P.layer_ops = reinterpret_cast<const uint32_t*>(ws + plan->off_layer_ops);
  P.layer_begin = reinterpret_cast<const uint32_t*>(ws + plan->off_layer_begin);
  P.nonroot = reinterpret_cast<const uint32_t*>(ws + plan->off_nonroot);
  P.aux = ws + plan->off_aux;
  P.dyn = dyn; P.ctrl = ctrl;
  P.prog_ops = reinterpret_cast<OpProg*>(ws + plan->off_prog_ops);
  P.prog_fields = reinterpret_cast<FieldProg*>(ws + plan->off_prog_fields);
  P.tile_cnt = reinterpret_cast<uint32_t*>(ws + g.off_tile_cnt);
  P.tile_base = reinterpret_cast<uint64_t*>(ws + g.off_tile_base);
  P.n_ops = n_ops; P.n_layers = h.n_layers; P.n_ragged = h.n_ragged;
  P.n_nonroot = static_cast<uint32_t>(h.nonroot_ops.size());
  P.n_tiles = g.n_tiles; P.n_fields = h.n_fields; P.count_fields = h.count_fields;
  P.waves_per_block = g.count_waves;
  P.lds_pad = plan->lds_pad;
  uint64_t* row_total = reinterpret_cast<uint64_t*>(ws + plan->off_row_total);

  // profiling events
  const uint32_t n_launch = h.n_layers == 0 ? 0 : (plan->fused ? 1 : h.n_layers);
  plan->n_tile_launches = n_launch;
  plan->tile_launch_layer.clear();
  const bool profile = plan->profile && !reg.own_tables;
  if (profile) {
    if (plan->timers.size() < 4 + n_launch) plan->timers.resize(4 + n_launch);
    for (Timer& t : plan->timers) {
      t.used = false;
      for (hipEvent_t& e : t.ev)
        if (!e) {
          hipError_t he = hipEventCreate(&e);
          if (he != hipSuccess) return hip_fail(plan, he, "hipEventCreate");
        }
    }
  }
  auto tick = [&](uint32_t which, int edge) {
    if (profile) {
      (void)hipEventRecord(plan->timers[which].ev[edge], st);
      plan->timers[which].used = true;
    }
  };
#define FBX_LAUNCH(expr, what)                                 \
  do {                                                         \
    hipError_t e_ = (expr);                                    \
    if (e_ != hipSuccess) return hip_fail(plan, e_, what);     \
  } while (0)

  const double compile_ms_before = plan->jit.compile_ms();
  // The tile kernel in one of its modes: the one compiled for this plan if the plan asks for
  // that and it can be had, else the generic one.
  auto tile_launch = [&](const TileParams& Q, int mode) -> hipError_t {
    if (plan->compile && !reg.own_tables)
      if (const FixedTileKernel* k = plan->jit.get(Q, mode, plan->host, plan->tile_threads, plan->lane_ops)) return launch_tile_fixed(*k, Q, st);
    return launch_tile(Q, mode, st);
  };
  // One attempt: everything is enqueued on the stream, then one synchronisation.
  auto run = [&](bool one) -> fbx_status {
    for (Timer& t : plan->timers) t.used = false;
    plan->tile_launch_layer.clear();
    FBX_LAUNCH(launch_reset(ctrl, g.arena_base, st), "reset");
    if (g.tile_engine) {
      // one workgroup per tile takes its records through every layer; offsets are checked tile by tile
      TileParams Q = g.tp;
      Q.raw = d_raw; Q.raw_len = raw_len; Q.rec_off = d_rec_off; Q.n_records = n_records;
      Q.prog = P.prog_ops;
      Q.lists = reinterpret_cast<const uint32_t*>(ws + plan->off_tile_lists);
      Q.list_begin = reinterpret_cast<const uint32_t*>(ws + plan->off_tile_list_begin);
      Q.rnr = reinterpret_cast<const uint32_t*>(ws + plan->off_rnr);
      Q.aux = P.aux; Q.ctrl = ctrl;
      Q.tile_cnt = P.tile_cnt; Q.tile_base = P.tile_base;
      Q.lb_state = nullptr; Q.row_cap = nullptr; Q.row_actual = nullptr;
      Q.n_ops = n_ops; Q.n_layers = h.n_layers; Q.n_ragged = h.n_ragged;
      Q.n_rnr = h.n_derive;
      Q.rnr_words = static_cast<uint32_t>(h.derive_tab.size());
      Q.alias_at = h.alias_at; Q.n_alias = h.n_alias;
      Q.n_lists = static_cast<uint32_t>(h.tile_list_begin.size()) - 1u;
      Q.aux_bytes = static_cast<uint32_t>(h.aux.size());

      Q.n_tiles = g.n_tiles; Q.n_fields = h.n_fields; Q.n_stage = h.n_stage;
      Q.lds_bytes = std::max(Q.lds_bytes, plan->lds_pad);
      Q.grid = plan->grid_limit;  // 0: as many persistent workgroups as run at the same time
      Q.spin_limit = plan->spin_limit;
      Q.prof = nullptr;
      Q.dbg = plan->dbg;
#ifdef FBX_TILE_PROF
      Q.prof = reinterpret_cast<uint64_t*>(ws + plan->off_prof);
      FBX_LAUNCH(hipMemsetAsync(Q.prof, 0, 32 * 8, st), "clearing phase counters");
#endif
      if (one) {
        // one launch: arrays sized from what the last call produced, bases found by look-back
        Q.row_cap = reinterpret_cast<const uint64_t*>(ws + plan->off_cap);
        Q.row_actual = reinterpret_cast<uint64_t*>(ws + plan->off_actual);
        Q.lb_state = P.tile_base;
        FBX_LAUNCH(hipMemcpyAsync(ws + plan->off_cap, plan->cap_host.data(), h.n_ragged * 8ull, hipMemcpyHostToDevice, st),
                   "capacity upload");
        tick(3, 0);
        FBX_LAUNCH(launch_alloc(P, Q.row_cap, ws_bytes, 0, st), "allocation kernel");
        tick(3, 1);
        if (plan->placement) FBX_LAUNCH(launch_fill64(Q.row_actual, h.n_ragged, 0, st), "running totals");
        else FBX_LAUNCH(launch_fill64(Q.lb_state, uint64_t(h.n_ragged) * g.n_tiles, 0, st), "look-back state");
        tick(4, 0);
        FBX_LAUNCH(tile_launch(Q, plan->placement ? 3 : 2), "tile kernel (one launch)");
        tick(4, 1);
        plan->tile_launch_layer.push_back(1);
      } else {
        if (h.n_ragged) {
          // the counting launch also needs the per-call programs: sizes are unknown, addresses unused
          FBX_LAUNCH(launch_programs(P, st), "program kernel");
          if (g.n_tiles) {
            tick(1, 0);
            FBX_LAUNCH(tile_launch(Q, 0), "tile kernel (counting)");
            tick(1, 1);
          }
          tick(2, 0);
          FBX_LAUNCH(launch_scan(P.tile_cnt, P.tile_base, row_total, reinterpret_cast<uint64_t*>(ws + g.off_scan_part), h.n_ragged, g.n_tiles, ctrl, st), "scan kernel");
          tick(2, 1);
        }
        tick(3, 0);
        FBX_LAUNCH(launch_alloc(P, row_total, ws_bytes, 0, st), "allocation kernel");
        tick(3, 1);
        if (g.n_tiles) {
          tick(4, 0);
          FBX_LAUNCH(tile_launch(Q, 1), "tile kernel");
          tick(4, 1);
          plan->tile_launch_layer.push_back(1);
        }
      }
    } else {
      tick(0, 0);
      FBX_LAUNCH(launch_validate(d_rec_off, n_records, raw_len, kTileLog2, ctrl, st), "validate");
      tick(0, 1);
      if (h.n_ragged) {
        if (g.n_tiles) {
          tick(1, 0);
          P.layer_lo = 1; P.layer_hi = h.n_layers;
          FBX_LAUNCH(launch_count(P, st), "count kernel");
          tick(1, 1);
        }
        tick(2, 0);
        FBX_LAUNCH(launch_scan(P.tile_cnt, P.tile_base, row_total, reinterpret_cast<uint64_t*>(ws + g.off_scan_part), h.n_ragged, g.n_tiles, ctrl, st), "scan kernel");
        tick(2, 1);
      }
      tick(3, 0);
      FBX_LAUNCH(launch_alloc(P, row_total, ws_bytes, plan->fused ? 0 : 1, st), "allocation kernel");
      tick(3, 1);
      if (g.n_tiles) {
        if (plan->fused) {
          P.layer_lo = 1; P.layer_hi = h.n_layers;
          tick(4, 0);
          FBX_LAUNCH(launch_walk(P, st), "walk kernel");
          tick(4, 1);
          plan->tile_launch_layer.push_back(1);
        } else {
          for (uint32_t l = 1; l <= h.n_layers; ++l) {
            P.layer_lo = P.layer_hi = l;
            tick(3 + l, 0);
            FBX_LAUNCH(launch_walk(P, st), "walk kernel");
            tick(3 + l, 1);
            plan->tile_launch_layer.push_back(l);
          }
        }
      }
    }
    FBX_LAUNCH(hipMemcpyAsync(plan->readback.data(), ws, plan->readback.size(), hipMemcpyDeviceToHost, st), "read-back");
    FBX_LAUNCH(hipStreamSynchronize(st), "synchronise");
#ifdef FBX_TILE_PROF
    if (g.tile_engine) {
      uint64_t pc[32];
      if (hipMemcpy(pc, ws + plan->off_prof, sizeof(pc), hipMemcpyDeviceToHost) == hipSuccess) {
        for (int k = 0; k < 2; ++k) {
          uint64_t sum = 0;
          for (int i = 0; i < 13; ++i) sum += pc[16 * k + i];
          fprintf(stderr, "[fbx prof] %s T=%u lds=%u grid-cycles=%llu :", k ? "write" : "count", 1u << g.tp.log2T,
                  g.tp.lds_bytes, (unsigned long long)sum);
          for (int i = 0; i < 13; ++i) fprintf(stderr, " p%d=%.1f%%", i, sum ? 100.0 * pc[16 * k + i] / sum : 0.0);
          fprintf(stderr, " placements=%llu windows=%llu polls=%llu", (unsigned long long)pc[16 * k + 15],
                  (unsigned long long)pc[16 * k + 13], (unsigned long long)pc[16 * k + 14]);
          fprintf(stderr, "\n");
        }
      }
    }
#endif
    return FBX_OK;
  };
  // Ragged arrays can be sized from what the last call produced (plus a margin): then the
  // counting launch is skipped.  A batch that does not fit its arrays, or a tile that needs
  // several passes, sends the call back to the exact sequence.
  // (every tile reads 512 bytes of placement words per ragged operator that is placed by look-back,
  // which those whose counts follow from another operator's are not: only worth it when that is
  // little next to the tile's own text)
  // (a batch with a tile that did not fit the LDS section is likely to be followed by more of its kind: the
  // sequence is then left untried for 1, 2, 4 ... up to 64 calls, so that such batches do not pay for two attempts each)
  const bool resting = plan->passes_skip > 0;
  if (resting) --plan->passes_skip;
  bool one = !resting && g.tile_engine && plan->one_launch && plan->learned && h.n_ragged && n_records && plan->learned_records &&
             ws_bytes > plan->margin_failed_ws &&
             (plan->placement || uint64_t(h.n_ragged - h.n_alias) * 512u * 2u <= (raw_len / n_records) << g.tp.log2T);
  if (one) {
    plan->cap_host.resize(h.n_ragged);
    for (uint32_t r = 0; r < h.n_ragged; ++r) {
      const unsigned __int128 scaled =
          (unsigned __int128)plan->learned_total[r] * n_records / plan->learned_records;
      // (a sixty-fourth, and sixteen standard deviations of a count that size: operators that yield signs for
      // few records, many at a time, vary far more between batches than their size suggests)
      const unsigned __int128 cap = scaled + scaled / 64 + (unsigned __int128)(16.0 * std::sqrt((double)scaled)) + 256;
      plan->cap_host[r] = cap > (unsigned __int128)(1ull << 60) ? (1ull << 60) : (uint64_t)cap;
    }
  }
  const Ctrl* c = reinterpret_cast<const Ctrl*>(plan->readback.data() + plan->off_ctrl);
  const char* fell_back = nullptr;
  for (;;) {
    fbx_status rs = run(one);
    if (rs != FBX_OK) return rs;
    if (!one && (c->err & CE_STALL)) {  // (only the one-launch sequence waits: this cannot happen)
      plan->error = "internal: a bounded wait between tiles ran out";
      return FBX_E_HIP;
    }
    if (one && (c->err & (CE_SPEC | CE_NOMEM | CE_STALL))) {
      // Every kernel has exited normally and the tiles that could not be placed wrote nothing: the
      // exact sequence (counting launch, scan, writing launch) can still answer the call.
      if (c->err & CE_PASSES) {
        plan->passes_backoff = plan->passes_backoff ? std::min(64u, plan->passes_backoff * 2u) : 1u;
        plan->passes_skip = plan->passes_backoff;
      }
      fell_back = (c->err & CE_STALL) ? "one-launch attempt fell back to the counting launch: a bounded wait for an earlier tile ran out"
                  : (c->err & CE_PASSES) ? "one-launch attempt fell back to the counting launch: a tile larger than the LDS section"
                  : (c->err & CE_SPEC) ? "one-launch attempt fell back to the counting launch: more signs than the arrays were sized for"
                                       : "one-launch attempt fell back to the counting launch: the margin on the arrays did not fit the workspace";
      if (!(c->err & (CE_SPEC | CE_STALL))) plan->margin_failed_ws = ws_bytes;
      one = false;  // fall back to counting first
      continue;
    }
    break;
  }
  plan->last_mode = one ? 2 : 1;
  if (one) plan->passes_backoff = 0;  // (the sequence went through: the next tile that does not fit starts over at one call)
  if (resting && !fell_back) fell_back = "one-launch sequence not tried: a recent batch had a tile larger than the LDS section";
#undef FBX_LAUNCH

  const OpDyn* y = reinterpret_cast<const OpDyn*>(plan->readback.data() + plan->off_dyn);
  if (c->err & CE_OFFSETS) {
    plan->error = "record offsets must be non-decreasing and end within raw_len";
    return FBX_E_INPUT;
  }
  if (c->err & CE_TILE) {
    plan->error = "a tile of records spans 2 GiB or more";
    return FBX_E_INPUT;
  }
  if (c->err & CE_OVERFLOW) {
    plan->error = "an operator produces 2^26 or more signs for one record";
    return FBX_E_INPUT;
  }
  if (c->err & CE_NOMEM) {
    if (reg.own_tables) {
      out->arena_high_water = c->required - g.arena_base;
      plan->error = "output buffer too small: need " + std::to_string(c->required - g.arena_base) + " bytes";
    } else {
      out->arena_high_water = c->required;
      plan->error = "workspace too small: need " + std::to_string(c->required) + " bytes";
    }
    return FBX_E_NOMEM;
  }
  const uint64_t* actual = reinterpret_cast<const uint64_t*>(plan->readback.data() + plan->off_actual);
  if (h.n_ragged && n_records) {  // remember the sizes for the next call
    plan->learned_total.resize(h.n_ragged);
    for (const HostOp& op : h.ops)
      if (!op.d.arity) {
        const size_t i = static_cast<size_t>(&op - h.ops.data());
        plan->learned_total[op.d.rag_row] = one ? actual[op.d.rag_row] : y[i].n_values;
      }
    plan->learned_records = n_records;
    plan->learned = true;
  }
  const bool arrival = one && plan->placement && h.n_ragged;
  uint64_t total = 0;
  for (size_t s = 0; s < plan->emitted.size(); ++s) {
    const uint32_t i = plan->emitted[s];
    const OpDesc& d = h.ops[i].d;
    fbx_slot_view& v = plan->slots[s];
    v.slot_id = h.ops[i].slot;
    v.fixed_arity = d.arity;
    v.n_values = (one && !d.arity) ? actual[d.rag_row] : y[i].n_values;
    v.values = reinterpret_cast<const uint64_t*>(reg.origin + y[i].values_off);
    v.offsets = d.arity ? nullptr : reinterpret_cast<const uint64_t*>(reg.origin + y[i].offsets_off);
    v.tile_ends = (arrival && !d.arity) ? P.tile_base + uint64_t(d.rag_row) * g.n_tiles : nullptr;
    total += v.n_values;
  }
  out->n_records = n_records;
  out->n_values_total = total;
  out->n_malformed_numeric = c->n_malformed;
  out->arena_high_water = reg.own_tables ? c->high_water - g.arena_base : c->high_water;
  out->n_slots = static_cast<uint32_t>(plan->slots.size());
  out->n_layers = h.n_layers;
  out->slots = plan->slots.data();
  plan->error = fell_back ? fell_back : "";  // (not an error: fbx_last_error doubles as a note after FBX_OK)
  if (plan->compile) {
    std::string note = plan->jit.note();
    if (plan->jit.compile_ms() > compile_ms_before) {
      char buf[96];
      snprintf(buf, sizeof buf, "compile=1: tile kernels compiled for this plan in %.0f ms", plan->jit.compile_ms() - compile_ms_before);
      note = note.empty() ? std::string(buf) : note + "; " + buf;
    }
    if (!note.empty()) plan->error += (plan->error.empty() ? "" : "; ") + note;
  }
  out->tile_launches = g.tile_engine ? (one ? 1u : (h.n_ragged ? 2u : 1u)) : 0u;
  out->arrival_tile_records = arrival ? 1u << g.tp.log2T : 0u;
  return FBX_OK;
}

}  // namespace

extern "C" {

fbx_status fbx_extract(fbx_plan* plan, const uint8_t* d_raw, uint64_t raw_len, const uint64_t* d_rec_off,
                       uint64_t n_records, void* hip_stream, fbx_result* out) {
  if (!plan || !out || !d_rec_off || (!d_raw && raw_len)) {
    if (plan) plan->error = "NULL argument";
    return FBX_E_ARG;
  }
  if (!plan->ws) { plan->error = "no workspace set"; return FBX_E_ARG; }
  if (n_records >= (1ull << 32)) { plan->error = "more than 2^32-1 records in one call"; return FBX_E_ARG; }
  const CallGeometry g = geometry(*plan, raw_len, n_records);
  if (g.arena_base > plan->ws_bytes) {
    out->arena_high_water = g.arena_base;
    plan->error = "workspace too small for the per-tile tables; need more than " + std::to_string(g.arena_base) + " bytes";
    return FBX_E_NOMEM;
  }
  const Regions reg{plan->ws, plan->ws_bytes, reinterpret_cast<uint64_t>(plan->ws), plan->ws_bytes, false};
  return extract_impl(plan, d_raw, raw_len, d_rec_off, n_records, hip_stream, out, reg, g);
}

// ---- the entry point that allocates nothing
// Its tables (control block, plan tables, per-call programs, per-tile counts, bases and look-back
// words) live in this array instead of a workspace.  Every GPU the library runs on holds its own
// copy from the moment the library is loaded there until the process ends.
}  // extern "C"

namespace {

constexpr uint64_t kScratchBytes = 64ull << 20;
static __device__ __align__(256) uint8_t scratch[kScratchBytes];
// (referenced by device code as well, so that the array is kept whatever the host side does with it)
__global__ void k_scratch_probe(uint8_t* out) { if (out) *out = scratch[0]; }

constexpr int kMaxDevices = 64;
struct ScratchOnDevice {
  uint8_t* ptr = nullptr;   // the array's address on that device (hipGetSymbolAddress, once)
  uint64_t owner = 0;       // id of the plan whose tables lie at its head
};
ScratchOnDevice g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

// The array's address on the current device, looked up once per device with that device current.
hipError_t scratch_on_current_device(int* dev_out, ScratchOnDevice** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  ScratchOnDevice& sd = g_scratch[dev];
  if (!sd.ptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    sd.ptr = static_cast<uint8_t*>(p);
  }
  *dev_out = dev;
  *out = &sd;
  return hipSuccess;
}

}  // namespace

extern "C" {

uint64_t fbx_static_scratch_bytes(void) { return kScratchBytes; }

fbx_status fbx_extract_static(fbx_plan* plan, const uint8_t* d_raw, uint64_t raw_len, const uint64_t* d_rec_off,
                              uint64_t n_records, void* d_out, uint64_t out_bytes, void* hip_stream, fbx_result* out) {
  if (!plan || !out || !d_rec_off || (!d_raw && raw_len) || !d_out) {
    if (plan) plan->error = "NULL argument";
    return FBX_E_ARG;
  }
  if (reinterpret_cast<uintptr_t>(d_out) & 255u) { plan->error = "the output buffer must be 256-byte aligned"; return FBX_E_ARG; }
  if (n_records >= (1ull << 32)) { plan->error = "more than 2^32-1 records in one call"; return FBX_E_ARG; }
  const CallGeometry g = geometry(*plan, raw_len, n_records);
  if (g.arena_base > kScratchBytes) {
    // (rejected before anything is enqueued: the tables of this batch do not fit the library's own array)
    out->arena_high_water = 0;
    plan->error = "this batch needs " + std::to_string(g.arena_base) + " bytes of tables (per tile and ragged operator); "
                  "the entry point that allocates nothing holds " + std::to_string(kScratchBytes) +
                  ": pass fewer records per call, or use fbx_extract with a workspace";
    return FBX_E_ARG;
  }
  int dev = 0;
  ScratchOnDevice* sd = nullptr;
  hipError_t e = scratch_on_current_device(&dev, &sd);
  if (e != hipSuccess) return hip_fail(plan, e, "address of the library's table array");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (sd->owner != plan->id) {  // another plan's tables (or none) lie there
    e = hipMemcpyAsync(sd->ptr, plan->tables.data(), plan->tables.size(), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);  // (the image is pageable host memory: done with it before returning)
    if (e != hipSuccess) { sd->owner = 0; return hip_fail(plan, e, "copying plan tables"); }
    sd->owner = plan->id;
  }
  const uint64_t origin = reinterpret_cast<uint64_t>(d_out) - g.arena_base;
  const Regions reg{sd->ptr, kScratchBytes, origin, g.arena_base + out_bytes, true};
  return extract_impl(plan, d_raw, raw_len, d_rec_off, n_records, hip_stream, out, reg, g);
}

fbx_status fbx_plan_kernel_ms(const fbx_plan* plan, uint32_t which, float* ms) {
  if (!plan || !ms) return FBX_E_ARG;
  auto one = [&](uint32_t idx, float& v) -> bool {
    if (idx >= plan->timers.size() || !plan->timers[idx].used) return false;
    return hipEventElapsedTime(&v, plan->timers[idx].ev[0], plan->timers[idx].ev[1]) == hipSuccess;
  };
  float v = 0.f;
  if (which < 4) {
    if (!one(which, v)) return FBX_E_ARG;
    *ms = v;
    return FBX_OK;
  }
  if (which == 4) {
    float sum = 0.f;
    for (uint32_t k = 0; k < plan->n_tile_launches; ++k) {
      if (!one(4 + k, v)) return FBX_E_ARG;
      sum += v;
    }
    *ms = sum;
    return FBX_OK;
  }
  if (which > 100 && which - 101 < plan->n_tile_launches) {
    if (!one(4 + (which - 101), v)) return FBX_E_ARG;
    *ms = v;
    return FBX_OK;
  }
  return FBX_E_ARG;
}

fbx_status fbx_arena_alloc(uint64_t* d_head, const uint64_t* d_sizes, uint64_t n, uint64_t* d_offsets,
                           uint32_t block_threads, void* hip_stream) {
  if (!d_head || (n && (!d_sizes || !d_offsets)) || block_threads < 64 || block_threads > 1024 || block_threads % 64 ||
      (n + block_threads - 1) / block_threads > 0x7fffffffull)
    return FBX_E_ARG;
  hipError_t e = launch_arena_alloc(d_head, d_sizes, n, d_offsets, block_threads, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FBX_OK : FBX_E_HIP;
}

fbx_status fbx_extract_unordered(fbx_plan* plan, uint32_t slot_id, const uint8_t* d_raw, uint64_t raw_len,
                                 const uint64_t* d_rec_off, uint64_t n_records, void* d_pool, uint64_t pool_bytes,
                                 uint64_t* d_state, int reset, uint64_t* d_thread_offsets, uint32_t* d_lengths,
                                 void* hip_stream, fbx_unordered_result* out) {
  if (!plan || !out || !d_rec_off || (!d_raw && raw_len) || !d_state || (n_records && (!d_thread_offsets || !d_lengths)) ||
      (!d_pool && pool_bytes)) {
    if (plan) plan->error = "NULL argument";
    return FBX_E_ARG;
  }
  if (!plan->ws) { plan->error = "no workspace set (the plan's tables are read from it)"; return FBX_E_ARG; }
  if ((reinterpret_cast<uintptr_t>(d_pool) & 127u) || n_records >= (1ull << 32)) {
    plan->error = "the pool must be 128-byte aligned and a call takes fewer than 2^32 records";
    return FBX_E_ARG;
  }
  const HostOp* found = nullptr;
  for (const HostOp& op : plan->host.ops)
    if ((op.d.flags & F_EMIT) && op.slot == slot_id) found = &op;
  if (!found || found->d.layer != 1 || found->d.arity != 0) {
    plan->error = "slot " + std::to_string(slot_id) + " is not an emitted operator of layer 1 with lists of varying length";
    return FBX_E_ARG;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  UnorderedParams U{};
  U.raw = d_raw; U.raw_len = raw_len; U.rec_off = d_rec_off; U.n_records = n_records;
  const OpDesc& d = found->d;
  U.op.kind = d.kind; U.op.flags = d.flags; U.op.arity = 0; U.op.rag_row = 0;
  U.op.aux_off = d.aux_off; U.op.aux_len = d.aux_len; U.op.a = U.op.b = 0;
  U.op.key = d.key; U.op.values = U.op.offsets = 0; U.op.field = d.field; U.op.stage = 0xffffffffu;
  U.aux = plan->ws + plan->off_aux;
  U.pool = static_cast<uint8_t*>(d_pool); U.pool_bytes = pool_bytes;
  U.state = d_state; U.thread_off = d_thread_offsets; U.lengths = d_lengths;
  hipError_t e;
  // the counters always start from zero; the head only when asked to (Section 5, "Reset GPU memory pool":
  // one store releases everything; without it this call allocates behind the calls before it)
  if (reset) e = launch_fill64(d_state, 4, 0, st);
  else e = launch_fill64(d_state + 1, 3, 0, st);
  if (e != hipSuccess) return hip_fail(plan, e, "resetting the pool's state");
  e = launch_unordered(U, st);
  if (e != hipSuccess) return hip_fail(plan, e, "kernel with in-kernel allocation");
  uint64_t state[4] = {0, 0, 0, 0};
  e = hipMemcpyAsync(state, d_state, sizeof state, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(plan, e, "read-back");
  out->n_values = state[2];
  out->n_malformed_numeric = state[3];
  out->pool_head = state[0];
  if (state[1] & CE_OFFSETS) { plan->error = "record offsets must be non-decreasing and end within raw_len"; return FBX_E_INPUT; }
  if (state[1] & CE_TILE) { plan->error = "a record spans 2 GiB or more"; return FBX_E_INPUT; }
  if (state[1] & CE_OVERFLOW) { plan->error = "an operator produces 2^26 or more signs for one record"; return FBX_E_INPUT; }
  if (state[1] & CE_NOMEM) {
    plan->error = "pool too small: " + std::to_string(state[0]) + " bytes would have sufficed";
    return FBX_E_NOMEM;
  }
  plan->error.clear();
  return FBX_OK;
}

fbx_status fbx_launch_overhead(uint32_t n_launches, void* hip_stream, double* microseconds) {
  if (!microseconds || n_launches == 0 || n_launches > 1000000u) return FBX_E_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (hipStreamSynchronize(st) != hipSuccess) { (void)hipGetLastError(); return FBX_E_HIP; }
  const auto t0 = std::chrono::steady_clock::now();
  hipError_t e = launch_empty(n_launches, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  const auto t1 = std::chrono::steady_clock::now();
  if (e != hipSuccess) { (void)hipGetLastError(); return FBX_E_HIP; }
  *microseconds = std::chrono::duration<double, std::micro>(t1 - t0).count();
  return FBX_OK;
}

fbx_status fbx_arena_reset(uint64_t* d_head, uint64_t value, void* hip_stream) {
  if (!d_head) return FBX_E_ARG;
  hipError_t e = launch_arena_reset(d_head, value, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FBX_OK : FBX_E_HIP;
}

}  // extern "C"
