// Kernel parameter block and launch wrappers shared by the kernels and the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include "fbx_internal.h"

namespace fbx {

constexpr int kBlock = 256;     // threads per workgroup of the walk, scan and allocation kernels
constexpr int kTileLog2 = 6;    // a tile is the 64 records one wavefront walks, one record per lane
constexpr int kTile = 1 << kTileLog2;

struct WalkParams {
  const uint8_t* raw;
  uint64_t raw_len;
  const uint64_t* rec_off;
  uint64_t n_records;
  uint64_t origin;  // address that array offsets (OpDyn) count from: the workspace base, or the address that
                    // puts the arena's first byte at the start of a caller's output buffer
  const OpDesc* ops;
  const FieldDesc* fields;
  const uint32_t* field_ops;
  const uint32_t* layer_ops;
  const uint32_t* layer_begin;
  const uint32_t* nonroot;
  const uint8_t* aux;
  OpDyn* dyn;
  OpProg* prog_ops;        // [n_ops], per call
  FieldProg* prog_fields;  // [n_fields], per call
  Ctrl* ctrl;
  uint32_t* tile_cnt;   // [n_ragged][n_tiles]
  uint64_t* tile_base;  // [n_ragged][n_tiles]
  uint32_t n_ops, n_layers, n_ragged, n_nonroot;
  uint32_t n_tiles, n_fields, count_fields;
  uint32_t layer_lo, layer_hi;  // 1-based, inclusive
  uint32_t waves_per_block;     // counting pass only
  uint32_t lds_pad;             // extra dynamic LDS per workgroup: lowers occupancy (tuning)
};

// ---- tile kernel: one workgroup takes a tile of 2^log2T records through every layer
// (512 lanes in the kernel for any plan; a kernel compiled for one plan may be compiled for 1024)
#ifndef FBX_TILE_THREADS
#define FBX_TILE_THREADS 512
#endif
constexpr int kTileThreads = FBX_TILE_THREADS;
constexpr uint32_t kRawPad = 16;  // first byte position of the staged raw text inside its LDS section

struct TileParams {
  const uint8_t* raw;
  uint64_t raw_len;
  const uint64_t* rec_off;
  uint64_t n_records;
  const OpProg* prog;          // [n_ops], per call (absolute addresses)
  const uint32_t* lists;       // work lists (operator indices, n_ops in all), then each operator's position in them
  const uint32_t* list_begin;  // TL_LAYER + 2 * (n_layers - 1) + 1 entries
  const uint32_t* rnr;         // how the counts of the ragged operators of layers >= 2 follow (PlanHost::derive_tab)
  const uint8_t* aux;
  Ctrl* ctrl;
  uint32_t* tile_cnt;          // [n_ragged][n_tiles], written by the counting launch
  const uint64_t* tile_base;   // [n_ragged][n_tiles], read by the writing launch
  uint64_t* lb_state;          // [n_ragged][n_tiles] look-back words (mode 2; shares the tile_base storage)
  const uint64_t* row_cap;     // [n_ragged] signs the arrays were sized for (mode 2)
  uint64_t* row_actual;        // [n_ragged] signs actually produced (mode 2)
  uint32_t n_ops, n_layers, n_ragged, n_rnr, n_lists, aux_bytes;  // (n_rnr: operators in rnr)
  uint32_t rnr_words;   // 32-bit words of the rnr table
  uint32_t alias_at;    // word of the rnr table at which the rows' (parent, scale, add) triples start
  uint32_t n_alias;     // ragged rows whose sign counts follow from another row's (PlanHost::n_alias)
  uint32_t n_mh;        // multi-valued hashes: the first n_mh entries of the ragged root list
  uint32_t n_split;     // multi-valued root operators of any kind: the first n_split entries of that list
  uint32_t n_gen;       // list operators of layers >= 2 (crosses and concats that are not computed along with their input)
  uint32_t n_tiles, n_fields, n_stage;
  uint32_t grid;        // upper limit of workgroups to launch (0: as many as run at the same time)
  uint32_t spin_limit;  // polls after which a wait for an earlier tile's count is given up (mode 2)
  uint32_t log2T;       // records per tile = 1 << log2T (at most 64)
  uint32_t raw_cap;     // bytes of raw text one pass of a workgroup can stage
  uint32_t row_stride;  // u16 entries per record in the field table (n_fields + 1, padded)
  // byte offsets of the LDS sections
  uint32_t o_off, o_rs, o_re, o_rows, o_raw, o_stage, o_cnt, o_start, o_run, o_base;
  uint32_t o_prog, o_lbeg, o_rnr, o_aux;  // plan tables
  uint32_t o_tot, o_ioff, o_ctab, o_cap, o_gfirst, o_gtot;
  uint32_t item_cap;    // comma positions kept per record and multi-valued hash
  uint32_t lds_bytes;
  uint64_t* prof;  // 32 phase counters (tuning builds only), else NULL
  uint32_t dbg;    // phases to leave out (tuning builds only; results are then wrong)
};

// One ragged root operator over a batch, allocating in the kernel (k_unordered).
struct UnorderedParams {
  const uint8_t* raw;
  uint64_t raw_len;
  const uint64_t* rec_off;
  uint64_t n_records;
  OpProg op;              // kind, flags, field, key, aux_off, aux_len are read
  const uint8_t* aux;     // the plan's table of bucket boundaries and prefixes
  uint8_t* pool;
  uint64_t pool_bytes;
  uint64_t* state;        // [4]: idle-memory head (bytes from the pool's base), error bits, signs, malformed numerics
  uint64_t* thread_off;   // [n_records] byte offset of a record's signs from the pool's base
  uint32_t* lengths;      // [n_records] signs of a record
};

// The fields of TileParams that the plan and the tile size fix (all but addresses, sizes of
// the batch and tuning switches): a kernel compiled for one plan has them as literals.
#define FBX_TILE_FIXED_FIELDS(X)                                                                                     \
  X(n_ops) X(n_layers) X(n_ragged) X(n_rnr) X(n_lists) X(aux_bytes) X(rnr_words) X(alias_at) X(n_alias) X(n_mh) X(n_split) X(n_gen) X(n_fields) \
  X(n_stage) X(log2T) X(raw_cap) X(row_stride) X(o_off) X(o_rs) X(o_re) X(o_rows) X(o_raw) X(o_stage) X(o_cnt)     \
  X(o_start) X(o_run) X(o_base) X(o_prog) X(o_lbeg) X(o_rnr) X(o_aux) X(o_tot) X(o_ioff) X(o_ctab) X(o_cap)         \
  X(o_gfirst) X(o_gtot) X(item_cap) X(lds_bytes)

#ifndef __HIPCC_RTC__  // (the launch wrappers are host code: not for the run-time compiler)
// mode 0: counting launch; 1: writing launch (bases from the scan over tiles);
// 2: counting and writing in one launch (bases by look-back, arrays sized by row_cap);
// 3: the same with bases by one atomic add per (ragged operator, tile) on row_actual: tiles in arrival order
hipError_t launch_tile(const TileParams& P, int mode, hipStream_t st);
hipError_t launch_fill64(uint64_t* p, uint64_t n, uint64_t value, hipStream_t st);
uint32_t tile_max_lds();  // dynamic LDS a workgroup of the tile kernel may ask for on this device

// A tile kernel compiled at run time for one plan, one tile shape and one mode.
struct FixedTileKernel {
  int mode = 0;
  std::vector<uint32_t> key;   // the values of FBX_TILE_FIXED_FIELDS it was compiled for
  void* module = nullptr;      // hipModule_t
  void* function = nullptr;    // hipFunction_t; null: the attempt failed
  uint32_t per_cu = 1;         // workgroups of it that fit a compute unit
  uint32_t threads = 512;      // lanes of a workgroup it was compiled for
  uint32_t lane_ops = 0;       // how tiles of 64 records run single-sign operators (FBX_LANE_OPS in fbx_tile.hip)
};
// The compiled kernels of one plan.
class TileJit {
 public:
  static constexpr size_t kMaxKernels = 12;
  TileJit() { kernels_.reserve(kMaxKernels); }
  ~TileJit();
  TileJit(const TileJit&) = delete;
  TileJit& operator=(const TileJit&) = delete;
  // The kernel for these parameters, compiled now if it is not there yet; null if there is none
  // (note() then says why).  The device the kernel is to run on must be current; h is the plan
  // the object belongs to (always the same one: its list bounds are compiled in too).
  const FixedTileKernel* get(const TileParams& P, int mode, const PlanHost& h, uint32_t threads, uint32_t lane_ops);
  void release();
  const std::string& note() const { return note_; }
  double compile_ms() const { return compile_ms_; }  // spent compiling so far
  uint32_t compiled() const { return compiled_; }
 private:
  std::vector<FixedTileKernel> kernels_;
  std::string note_;
  double compile_ms_ = 0;
  uint32_t compiled_ = 0;
};
hipError_t launch_tile_fixed(const FixedTileKernel& k, const TileParams& P, hipStream_t st);
// The text that TileJit compiles for these parameters (fbx_tile.hip behind a few definitions).
std::string tile_kernel_source(const TileParams& P, int mode, const PlanHost& h, uint32_t threads, uint32_t lane_ops);
uint32_t tile_cu_count();

hipError_t launch_reset(Ctrl* ctrl, uint64_t arena_base, hipStream_t st);
hipError_t launch_validate(const uint64_t* rec_off, uint64_t n_records, uint64_t raw_len, uint32_t log2T, Ctrl* ctrl,
                           hipStream_t st);
hipError_t launch_count(const WalkParams& P, hipStream_t st);
hipError_t launch_walk(const WalkParams& P, hipStream_t st);
// part: n_ragged * scan_segments(n_tiles) words of scratch (the sums of the segments a row is cut into)
constexpr uint32_t kScanSeg = 4096;  // tiles a workgroup of the scan kernels takes
uint32_t scan_segments(uint32_t n_tiles);
hipError_t launch_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total, uint64_t* part, uint32_t n_ragged,
                       uint32_t n_tiles, const Ctrl* ctrl, hipStream_t st);
hipError_t launch_alloc(const WalkParams& P, const uint64_t* row_total, uint64_t ws_bytes, int reuse, hipStream_t st);
hipError_t launch_programs(const WalkParams& P, hipStream_t st);
hipError_t launch_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets, uint32_t threads,
                              hipStream_t st);
hipError_t launch_arena_reset(uint64_t* head, uint64_t value, hipStream_t st);
hipError_t launch_unordered(const UnorderedParams& U, hipStream_t st);
hipError_t launch_empty(uint32_t n, hipStream_t st);  // n launches of an empty kernel with five pointer arguments
#endif  // __HIPCC_RTC__

}  // namespace fbx
