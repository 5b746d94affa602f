// Internal declarations shared by the host side and the HIP kernels of libfbx.
// Nothing here is part of the C ABI.
#pragma once

#include <stdint.h>

#include <string>
#include <vector>

#include "fbx.h"

namespace fbx {

enum OpKind : uint32_t { OP_HASH = 1, OP_NGRAM = 2, OP_BUCKET = 3, OP_FILTER = 4, OP_CROSS = 5, OP_CONCAT = 6 };

enum OpFlags : uint32_t {
  F_MULTI = 1u,
  F_EMIT = 2u,
  F_STREAM = 4u,  // tile kernel: no later operator reads the signs from memory (they are only the caller's)
  F_NEVER = 8u    // a multi-valued filter whose prefix holds a comma: no token can begin with it
};

// Device-visible operator descriptor (64 bytes).  Filled once at plan time.
struct OpDesc {
  uint32_t kind;
  uint32_t flags;
  uint32_t field;    // root operators: positional field index
  uint32_t arity;    // signs per record when fixed, 0 when ragged
  uint32_t a, b;     // cross / concat: input operator indices
  uint32_t aux_off;  // byte offset into the aux table (bucket bounds, filter prefix)
  uint32_t aux_len;  // #bounds, prefix length, or n-gram width
  uint64_t key;      // hash/ngram/filter: FNV state after the 8 seed bytes;
                     // cross/bucket: slot key mix64(seed)
  uint32_t rag_row;  // row among ragged operators (count tables), 0xffffffff if fixed
  uint32_t layer;    // 1-based
  uint32_t birth;    // == layer
  uint32_t death;    // last layer that reads this operator's output (>= layer)
  uint32_t stage;    // row of the on-chip sign table (single-sign operators that feed a later
                     // operator), 0xffffffff if none
  uint32_t fuse;     // tile kernel.  A cross of a multi-valued hash with a single sign is computed
                     // by the lane that hashes the item: 1 when the hash is input a, 2 when it is
                     // input b, 0 for every other cross.  For the multi-valued hash itself: first
                     // entry (low 16 bits) and number (high 16 bits) of such crosses in
                     // PlanHost::derive_tab's list of them.
};
static_assert(sizeof(OpDesc) == 64, "OpDesc must stay 64 bytes");

// Per-field program: which root operators read field k.
enum FieldClass : uint32_t {
  FC_SKIP = 0,    // no operator reads the field: only its end is looked for
  FC_HASH1 = 1,   // exactly one operator, a single-valued hash: hashed while its tab is looked for
  FC_GENERIC = 2  // anything else: find the end, then run every operator on the span
};
struct FieldDesc {
  uint32_t op_begin;   // into the field_ops table
  uint32_t op_count;
  uint32_t cls;        // FieldClass
  uint32_t need;       // bit 0: some operator needs the comma count of the field
};
static_assert(sizeof(FieldDesc) == 16, "FieldDesc must stay 16 bytes");

// Per-call flattened programs, written by the allocation kernel once the
// operators' arrays are placed: everything the walk needs about an operator (or
// about a single-valued hash field) in one aligned record, so that one scalar
// load per step replaces a chain of dependent table lookups.
struct OpProg {
  uint32_t kind, flags, arity, rag_row;
  uint32_t aux_off, aux_len, a, b;
  uint64_t key;
  uint64_t values;   // absolute device address of the values array
  uint64_t offsets;  // absolute device address of the offsets array (ragged only)
  uint32_t field;    // root operators: positional field index
  uint32_t stage;    // row of the on-chip sign table, 0xffffffff if none
};
static_assert(sizeof(OpProg) == 64, "OpProg must stay 64 bytes");
struct FieldProg {
  uint32_t cls, need, op_begin, op_count;
  uint64_t key;      // FC_HASH1: FNV state after the seed bytes
  uint64_t dst;      // FC_HASH1: absolute device address of the values array
};
static_assert(sizeof(FieldProg) == 32, "FieldProg must stay 32 bytes");

// Per-call, per-operator placement, written by the allocation kernel.
struct OpDyn {
  uint64_t values_off;   // byte offset of the values array from the workspace base
  uint64_t offsets_off;  // byte offset of the offsets array (ragged only)
  uint64_t n_values;
  uint64_t pad;
};

// Device control block at the head of the workspace (read back once per call).
struct Ctrl {
  uint32_t err;            // bit 0 bad offsets, bit 1 out of memory, bit 2 count overflow, bit 3 tile too long
  uint32_t pad0;
  uint64_t required;       // workspace bytes needed (valid when the allocation kernel ran)
  uint64_t head;           // idle-memory head of the arena (byte offset from workspace base)
  uint64_t high_water;
  uint64_t n_malformed;
  uint64_t max_tile_bytes;
  uint64_t slow_tiles;     // tiles that did not fit the staged fast path
  uint32_t ticket[2];      // next tile of the tile kernel's counting / writing launch
};
static_assert(sizeof(Ctrl) == 64, "Ctrl must stay 64 bytes");

enum CtrlErr : uint32_t {
  CE_OFFSETS = 1u, CE_NOMEM = 2u, CE_OVERFLOW = 4u, CE_TILE = 8u,
  CE_SPEC = 16u,   // one-launch mode cannot place this batch (capacity or tile size): run the counting launch
  CE_STALL = 32u,  // a bounded wait in the one-launch mode ran out
  CE_PASSES = 64u  // (with CE_SPEC) the reason was a tile whose text does not fit the LDS section
};

struct HostOp {
  std::string id;
  OpDesc d{};
  uint32_t slot = 0;
  uint64_t seed = 0;
  std::vector<int64_t> bounds;
  std::vector<uint8_t> prefix;
};

// Parsed, layered plan (host).  Built by parse_plan(); no HIP calls involved.
struct PlanHost {
  uint32_t n_fields = 0;
  uint32_t n_layers = 0;
  uint32_t n_ragged = 0;
  std::vector<HostOp> ops;             // spec order
  std::vector<uint32_t> layer_ops;     // operator indices grouped by layer
  std::vector<uint32_t> layer_begin;   // n_layers + 1 entries into layer_ops
  std::vector<uint32_t> nonroot_ops;   // operators of layers >= 2, in spec order
  std::vector<uint8_t> aux;            // bounds (8-byte aligned) and prefixes
  std::vector<FieldDesc> fields;       // n_fields entries
  std::vector<uint32_t> field_ops;     // root operator indices grouped by field, spec order inside a field
  uint32_t count_fields = 0;           // the counting pass may stop after this many fields
  // Work lists of the tile kernel: operator indices grouped by how a tile of
  // records runs them.  List ids: see TileList.
  std::vector<uint32_t> tile_lists;       // the lists one after the other (n_ops entries), then for every
                                          // operator its position in that sequence (n_ops entries)
  std::vector<uint32_t> tile_list_begin;  // n_tile_lists + 1 entries into tile_lists
  uint32_t n_stage = 0;                   // rows of the on-chip sign table
  // Counts of the ragged operators of layers >= 2 follow from their inputs' counts.  Table of
  // 32-bit words: a header of 4 * ceil(n_layers / 4) words (word l - 2 = first entry of layer l,
  // for l = 2 .. n_layers + 1), then four words per operator, layer after layer: row of the
  // result, input a, input b (a row of the count table, or 0x80000000 | arity for an input
  // of fixed arity), and 0 for a cross (counts multiply) or 1 for a concat (counts add).
  // After these, one word per cross that is computed along with its multi-valued hash (see
  // OpDesc::fuse): its position in tile_lists, grouped by hash.
  std::vector<uint32_t> derive_tab;
  uint32_t n_derive = 0;                  // operators in derive_tab
  uint32_t alias_at = 0, n_alias = 0;     // derive_tab[alias_at + 3 * row ..]: (parent row or kNoAlias, scale, add); rows that have a parent
};

// Work lists of the tile kernel.  Layer 1 has four lists; TL_FUSED holds the crosses that
// the lanes of a multi-valued hash compute along with its items; every later layer l
// has two, TL_LAYER + 2 * (l - 2) (crosses of two single signs) and the next
// one (every other cross or concat).
constexpr uint32_t kNoAlias = 0xffffffffu;  // a ragged row whose sign counts follow from no other row's (PlanHost::alias_at)
enum TileList : uint32_t { TL_HASH1 = 0, TL_BUCKET1 = 1, TL_RAGROOT = 2, TL_NGRAM = 3, TL_FUSED = 4, TL_LAYER = 5 };

// Returns FBX_OK or FBX_E_SPEC (message in err).
fbx_status parse_plan(const char* spec, size_t len, PlanHost& out, std::string& err);

}  // namespace fbx
