// Host-side planning: spec text -> typed operator list -> layers -> device tables.
//
// The paper fixes the operator order once, before any batch is processed
// (Section 4, "Inner-GPU operator launching"), from the operators' dependency
// graph: operators without dependencies make up the first layer and every
// other operator is placed by its depth below them, so that operators of one
// layer are mutually independent (Section 4, "Scheduling").  This file does
// that planning; it makes no HIP call and works on a machine without a GPU.
#include <algorithm>
#include <cstring>
#include <sstream>
#include <unordered_map>

#include "fbx_internal.h"

namespace fbx {
namespace {

constexpr uint64_t kFnvBasis = 0xcbf29ce484222325ull;
constexpr uint64_t kFnvPrime = 0x100000001b3ull;

// FNV-1a state after absorbing the seed's eight little-endian bytes: token
// hashing then continues from here, so seeding costs nothing per token.
uint64_t seeded_state(uint64_t seed) {
  uint64_t h = kFnvBasis;
  for (int i = 0; i < 8; ++i) {
    h ^= (seed >> (8 * i)) & 0xffu;
    h *= kFnvPrime;
  }
  return h;
}

uint64_t mix64_host(uint64_t x) {
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

bool to_u64(const std::string& s, uint64_t& v) {
  if (s.empty() || s.size() > 20) return false;
  unsigned __int128 acc = 0;
  for (char c : s) {
    if (c < '0' || c > '9') return false;
    acc = acc * 10 + static_cast<unsigned>(c - '0');
    if (acc > UINT64_MAX) return false;
  }
  v = static_cast<uint64_t>(acc);
  return true;
}

bool to_i64(const std::string& s, int64_t& v) {
  bool neg = !s.empty() && s[0] == '-';
  uint64_t mag;
  if (!to_u64(neg ? s.substr(1) : s, mag)) return false;
  if (neg) {
    if (mag > (1ull << 63)) return false;
    v = static_cast<int64_t>(0 - mag);
  } else {
    if (mag > static_cast<uint64_t>(INT64_MAX)) return false;
    v = static_cast<int64_t>(mag);
  }
  return true;
}

bool valid_id(const std::string& s) {
  if (s.empty() || s.size() > 63) return false;
  return std::all_of(s.begin(), s.end(), [](char c) {
    return (c >= '0' && c <= '9') || (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_';
  });
}

int hex_digit(char c) {
  if (c >= '0' && c <= '9') return c - '0';
  if (c >= 'a' && c <= 'f') return c - 'a' + 10;
  if (c >= 'A' && c <= 'F') return c - 'A' + 10;
  return -1;
}

std::vector<std::string> split_ws(const std::string& line) {
  std::vector<std::string> out;
  size_t i = 0;
  while (i < line.size()) {
    while (i < line.size() && (line[i] == ' ' || line[i] == '\r')) ++i;
    size_t j = i;
    while (j < line.size() && line[j] != ' ' && line[j] != '\r') ++j;
    if (j > i) out.emplace_back(line.substr(i, j - i));
    i = j;
  }
  return out;
}

struct KindInfo {
  const char* name;
  OpKind kind;
  std::vector<const char*> keys;  // exactly these keys, each once
};

const KindInfo kKinds[] = {
    {"hash", OP_HASH, {"slot", "seed", "emit", "field", "multi"}},
    {"ngram", OP_NGRAM, {"slot", "seed", "emit", "field", "n"}},
    {"bucket", OP_BUCKET, {"slot", "seed", "emit", "field", "multi", "bounds"}},
    {"filter", OP_FILTER, {"slot", "seed", "emit", "field", "multi", "prefix"}},
    {"cross", OP_CROSS, {"slot", "seed", "emit", "a", "b"}},
    {"concat", OP_CONCAT, {"slot", "emit", "a", "b"}},
};

}  // namespace

fbx_status parse_plan(const char* spec, size_t len, PlanHost& plan, std::string& err) {
  plan = PlanHost{};
  std::string text(spec, len);
  if (text.find('\0') != std::string::npos) {
    err = "spec contains a NUL byte";
    return FBX_E_SPEC;
  }
  std::unordered_map<std::string, uint32_t> by_id;
  std::unordered_map<uint32_t, uint32_t> emitted_slot;
  std::istringstream in(text);
  std::string line;
  int lineno = 0, stage = 0;
  auto fail = [&](const std::string& what) {
    err = "line " + std::to_string(lineno) + ": " + what;
    return FBX_E_SPEC;
  };
  while (std::getline(in, line)) {
    ++lineno;
    std::vector<std::string> tok = split_ws(line);
    if (tok.empty() || tok[0][0] == '#') continue;
    if (stage == 0) {
      if (tok.size() != 2 || tok[0] != "fbx" || tok[1] != "1") return fail("expected 'fbx 1'");
      stage = 1;
      continue;
    }
    if (stage == 1) {
      uint64_t f = 0;
      if (tok.size() != 2 || tok[0] != "fields" || !to_u64(tok[1], f) || f < 1 || f > 65535)
        return fail("expected 'fields <1..65535>'");
      plan.n_fields = static_cast<uint32_t>(f);
      stage = 2;
      continue;
    }
    if (tok[0] != "op" || tok.size() < 3) return fail("expected 'op <id> <kind> key=value ...'");
    if (!valid_id(tok[1])) return fail("bad operator id '" + tok[1] + "'");
    if (by_id.count(tok[1])) return fail("duplicate operator id '" + tok[1] + "'");
    if (plan.ops.size() >= 65535) return fail("too many operators");
    const KindInfo* ki = nullptr;
    for (const KindInfo& k : kKinds)
      if (tok[2] == k.name) ki = &k;
    if (!ki) return fail("unknown operator kind '" + tok[2] + "'");

    std::unordered_map<std::string, std::string> kv;
    for (size_t i = 3; i < tok.size(); ++i) {
      size_t eq = tok[i].find('=');
      if (eq == std::string::npos) return fail("expected key=value, got '" + tok[i] + "'");
      std::string key = tok[i].substr(0, eq);
      bool known = false;
      for (const char* k : ki->keys) known |= key == k;
      if (!known) return fail("key '" + key + "' does not belong to a " + ki->name + " operator");
      if (!kv.emplace(key, tok[i].substr(eq + 1)).second) return fail("key '" + key + "' given twice");
    }
    for (const char* k : ki->keys)
      if (!kv.count(k)) return fail(std::string("missing key '") + k + "'");

    HostOp op;
    op.id = tok[1];
    op.d.kind = ki->kind;
    op.d.rag_row = 0xffffffffu;
    uint64_t u = 0;
    if (!to_u64(kv["slot"], u) || u > 0xffffffffull) return fail("bad slot");
    op.slot = static_cast<uint32_t>(u);
    if (!to_u64(kv["emit"], u) || u > 1) return fail("emit must be 0 or 1");
    if (u) op.d.flags |= F_EMIT;
    if (ki->kind != OP_CONCAT) {
      if (!to_u64(kv["seed"], op.seed)) return fail("bad seed");
    }
    const bool root = ki->kind != OP_CROSS && ki->kind != OP_CONCAT;
    if (root) {
      if (!to_u64(kv["field"], u) || u >= plan.n_fields) return fail("field index out of range");
      op.d.field = static_cast<uint32_t>(u);
      if (ki->kind != OP_NGRAM) {
        if (!to_u64(kv["multi"], u) || u > 1) return fail("multi must be 0 or 1");
        if (u) op.d.flags |= F_MULTI;
      }
      op.d.layer = 1;
    }
    switch (ki->kind) {
      case OP_HASH:
        op.d.key = seeded_state(op.seed);
        op.d.arity = (op.d.flags & F_MULTI) ? 0 : 1;
        break;
      case OP_NGRAM:
        if (!to_u64(kv["n"], u) || u < 1 || u > 8) return fail("n must be in 1..8");
        op.d.aux_len = static_cast<uint32_t>(u);
        op.d.key = seeded_state(op.seed);
        op.d.arity = 0;
        break;
      case OP_FILTER: {
        const std::string& hx = kv["prefix"];
        if (hx.size() % 2 || hx.size() / 2 > 255) return fail("prefix must be an even number of hex digits (<= 255 bytes)");
        for (size_t i = 0; i < hx.size(); i += 2) {
          int hi = hex_digit(hx[i]), lo = hex_digit(hx[i + 1]);
          if (hi < 0 || lo < 0) return fail("prefix is not hex");
          op.prefix.push_back(static_cast<uint8_t>(hi * 16 + lo));
        }
        op.d.aux_len = static_cast<uint32_t>(op.prefix.size());
        op.d.key = seeded_state(op.seed);
        op.d.arity = 0;
        break;
      }
      case OP_BUCKET: {
        const std::string& bs = kv["bounds"];
        size_t pos = 0;
        while (!bs.empty()) {
          size_t comma = bs.find(',', pos);
          std::string item = bs.substr(pos, comma == std::string::npos ? std::string::npos : comma - pos);
          int64_t b;
          if (!to_i64(item, b)) return fail("bad boundary '" + item + "'");
          if (!op.bounds.empty() && b < op.bounds.back()) return fail("boundaries must be non-decreasing");
          op.bounds.push_back(b);
          if (op.bounds.size() > 4096) return fail("more than 4096 boundaries");
          if (comma == std::string::npos) break;
          pos = comma + 1;
        }
        op.d.aux_len = static_cast<uint32_t>(op.bounds.size());
        op.d.key = mix64_host(op.seed);
        op.d.arity = (op.d.flags & F_MULTI) ? 0 : 1;
        break;
      }
      case OP_CROSS:
      case OP_CONCAT: {
        auto ia = by_id.find(kv["a"]), ib = by_id.find(kv["b"]);
        // only earlier lines are visible, which rules out forward and self references (cycles)
        if (ia == by_id.end() || ib == by_id.end()) return fail("input names no earlier operator");
        op.d.a = ia->second;
        op.d.b = ib->second;
        const OpDesc& da = plan.ops[op.d.a].d;
        const OpDesc& db = plan.ops[op.d.b].d;
        op.d.layer = 1 + std::max(da.layer, db.layer);
        uint64_t k = 0;
        if (da.arity && db.arity)
          k = ki->kind == OP_CROSS ? uint64_t(da.arity) * db.arity : uint64_t(da.arity) + db.arity;
        // a fixed arity at or beyond the per-record sign limit could never be produced (and arities of
        // 2^31 and more would collide with the flag bit of the derived-count table)
        if (k >= (1ull << 26)) return fail("operator would produce 2^26 or more signs for every record");
        op.d.arity = static_cast<uint32_t>(k);
        if (ki->kind == OP_CROSS) op.d.key = mix64_host(op.seed);
        break;
      }
    }
    if (op.d.flags & F_EMIT) {
      if (!emitted_slot.emplace(op.slot, 0).second) return fail("slot " + std::to_string(op.slot) + " is emitted twice");
    }
    op.d.birth = op.d.death = op.d.layer;
    by_id.emplace(op.id, static_cast<uint32_t>(plan.ops.size()));
    plan.ops.push_back(std::move(op));
  }
  if (stage < 2) {
    err = "spec needs 'fbx 1' and 'fields <F>' lines";
    return FBX_E_SPEC;
  }

  // Layers, liveness, ragged rows, aux table.
  for (HostOp& op : plan.ops) plan.n_layers = std::max(plan.n_layers, op.d.layer);
  for (HostOp& op : plan.ops) {
    if (op.d.kind == OP_CROSS || op.d.kind == OP_CONCAT) {
      plan.ops[op.d.a].d.death = std::max(plan.ops[op.d.a].d.death, op.d.layer);
      plan.ops[op.d.b].d.death = std::max(plan.ops[op.d.b].d.death, op.d.layer);
    }
  }
  plan.layer_begin.assign(plan.n_layers + 1, 0);
  for (uint32_t l = 1; l <= plan.n_layers; ++l) {
    plan.layer_begin[l - 1] = static_cast<uint32_t>(plan.layer_ops.size());
    // keep operators of one kind next to each other so that neighbouring lanes
    // of a wavefront mostly run the same code
    std::vector<uint32_t> ids;
    for (uint32_t i = 0; i < plan.ops.size(); ++i)
      if (plan.ops[i].d.layer == l) ids.push_back(i);
    std::stable_sort(ids.begin(), ids.end(), [&](uint32_t x, uint32_t y) {
      const OpDesc& a = plan.ops[x].d;
      const OpDesc& b = plan.ops[y].d;
      if (a.kind != b.kind) return a.kind < b.kind;
      return (a.flags & F_MULTI) < (b.flags & F_MULTI);
    });
    plan.layer_ops.insert(plan.layer_ops.end(), ids.begin(), ids.end());
  }
  plan.layer_begin[plan.n_layers] = static_cast<uint32_t>(plan.layer_ops.size());
  // Rows of the ragged operators: those of the last layer (if it is not the first) come last, in
  // spec order, because the tile kernel derives their counts in the same step that scans them.
  for (int last = 0; last < 2; ++last)
    for (HostOp& op : plan.ops)
      if (op.d.arity == 0 && (op.d.layer > 1 && op.d.layer == plan.n_layers) == (last == 1)) op.d.rag_row = plan.n_ragged++;
  for (uint32_t i = 0; i < plan.ops.size(); ++i) {
    OpDesc& d = plan.ops[i].d;
    if (d.layer > 1) plan.nonroot_ops.push_back(i);
    if (d.kind == OP_BUCKET) {
      while (plan.aux.size() % 8) plan.aux.push_back(0);
      d.aux_off = static_cast<uint32_t>(plan.aux.size());
      const uint8_t* p = reinterpret_cast<const uint8_t*>(plan.ops[i].bounds.data());
      plan.aux.insert(plan.aux.end(), p, p + plan.ops[i].bounds.size() * 8);
    } else if (d.kind == OP_FILTER) {
      d.aux_off = static_cast<uint32_t>(plan.aux.size());
      plan.aux.insert(plan.aux.end(), plan.ops[i].prefix.begin(), plan.ops[i].prefix.end());
    }
  }
  while (plan.aux.size() % 16) plan.aux.push_back(0);
  // field programs: the root operators of every field, and how the field is walked
  plan.fields.assign(plan.n_fields, FieldDesc{0, 0, FC_SKIP, 0});
  for (uint32_t k = 0; k < plan.n_fields; ++k) {
    FieldDesc& f = plan.fields[k];
    f.op_begin = static_cast<uint32_t>(plan.field_ops.size());
    for (uint32_t i = 0; i < plan.ops.size(); ++i) {
      const OpDesc& d = plan.ops[i].d;
      if (d.layer != 1 || d.field != k) continue;
      plan.field_ops.push_back(i);
      ++f.op_count;
      if ((d.kind == OP_HASH || d.kind == OP_BUCKET) && (d.flags & F_MULTI)) f.need |= 1u;
      if (d.arity == 0) plan.count_fields = k + 1;
    }
    if (f.op_count == 0) f.cls = FC_SKIP;
    else if (f.op_count == 1 && plan.ops[plan.field_ops[f.op_begin]].d.kind == OP_HASH &&
             !(plan.ops[plan.field_ops[f.op_begin]].d.flags & F_MULTI)) f.cls = FC_HASH1;
    else f.cls = FC_GENERIC;
  }
  if (plan.n_ragged > 512) {
    err = "more than 512 ragged operators";
    return FBX_E_SPEC;
  }
  // Tile kernel: single-sign operators that feed a later operator keep their
  // signs on chip (one table row each); work lists group operators by the code
  // that runs them, layer by layer.
  for (HostOp& op : plan.ops) { op.d.stage = 0xffffffffu; op.d.fuse = 0; }
  for (const HostOp& op : plan.ops) {
    if (op.d.kind != OP_CROSS && op.d.kind != OP_CONCAT) continue;
    for (uint32_t in : {op.d.a, op.d.b}) {
      OpDesc& di = plan.ops[in].d;
      if (di.arity == 1 && di.stage == 0xffffffffu) di.stage = plan.n_stage++;
    }
  }
  const uint32_t n_lists = TL_LAYER + (plan.n_layers > 1 ? 2 * (plan.n_layers - 1) : 0);
  std::vector<std::vector<uint32_t>> lists(n_lists);
  for (uint32_t i = 0; i < plan.ops.size(); ++i) {
    const OpDesc& d = plan.ops[i].d;
    if (d.layer == 1) {
      if (d.kind == OP_NGRAM) lists[TL_NGRAM].push_back(i);
      else if (d.arity == 0) lists[TL_RAGROOT].push_back(i);
      else if (d.kind == OP_HASH) lists[TL_HASH1].push_back(i);
      else lists[TL_BUCKET1].push_back(i);
    } else {
      const bool single = d.kind == OP_CROSS && plan.ops[d.a].d.arity == 1 && plan.ops[d.b].d.arity == 1;
      auto multi_hash = [&](uint32_t in) {
        const OpDesc& di = plan.ops[in].d;
        return di.layer == 1 && di.kind == OP_HASH && di.arity == 0;
      };
      uint32_t fuse = 0;
      if (d.kind == OP_CROSS && multi_hash(d.a) && plan.ops[d.b].d.arity == 1) fuse = 1;
      if (d.kind == OP_CROSS && multi_hash(d.b) && plan.ops[d.a].d.arity == 1) fuse = 2;
      plan.ops[i].d.fuse = fuse;
      if (fuse) lists[TL_FUSED].push_back(i);
      else lists[TL_LAYER + 2 * (d.layer - 2) + (single ? 0 : 1)].push_back(i);
    }
  }
  // neighbouring lanes run neighbouring list entries: keep like with like.  Multi-valued hashes
  // come first, then the other multi-valued operators, then the single-valued filters.
  auto root_class = [&](uint32_t x) {
    const OpDesc& d = plan.ops[x].d;
    return d.kind == OP_HASH ? 0u : ((d.flags & F_MULTI) ? 1u : 2u);
  };
  std::stable_sort(lists[TL_RAGROOT].begin(), lists[TL_RAGROOT].end(), [&](uint32_t x, uint32_t y) {
    return root_class(x) != root_class(y) ? root_class(x) < root_class(y) : plan.ops[x].d.kind < plan.ops[y].d.kind;
  });
  for (HostOp& op : plan.ops) {
    OpDesc& d = op.d;
    if (d.kind == OP_FILTER && (d.flags & F_MULTI) && d.aux_len &&
        std::memchr(plan.aux.data() + d.aux_off, ',', d.aux_len))
      d.flags |= F_NEVER;
  }
  for (const std::vector<uint32_t>& l : lists) {
    plan.tile_list_begin.push_back(static_cast<uint32_t>(plan.tile_lists.size()));
    plan.tile_lists.insert(plan.tile_lists.end(), l.begin(), l.end());
  }
  plan.tile_list_begin.push_back(static_cast<uint32_t>(plan.tile_lists.size()));
  // whose signs does a later operator of the tile kernel read from memory?  (single signs are
  // read from the on-chip table, a multi-valued hash's items by the lanes that compute them)
  for (HostOp& op : plan.ops) op.d.flags |= F_STREAM;
  for (const HostOp& op : plan.ops) {
    if (op.d.kind != OP_CROSS && op.d.kind != OP_CONCAT) continue;
    if (plan.ops[op.d.a].d.arity != 1 && op.d.fuse != 1) plan.ops[op.d.a].d.flags &= ~(uint32_t)F_STREAM;
    if (plan.ops[op.d.b].d.arity != 1 && op.d.fuse != 2) plan.ops[op.d.b].d.flags &= ~(uint32_t)F_STREAM;
  }
  {  // every operator is in exactly one list: append where each one went
    const size_t n = plan.ops.size();
    plan.tile_lists.resize(2 * n);
    for (uint32_t pos = 0; pos < n; ++pos) plan.tile_lists[n + plan.tile_lists[pos]] = pos;
  }
  if (plan.n_layers > 1) {
    const uint32_t hw = 4u * ((plan.n_layers + 3u) / 4u);
    plan.derive_tab.assign(hw, 0u);
    for (uint32_t layer = 2; layer <= plan.n_layers; ++layer) {
      plan.derive_tab[layer - 2] = plan.n_derive;
      for (uint32_t i : plan.nonroot_ops) {  // (spec order inside a layer)
        const OpDesc& d = plan.ops[i].d;
        if (d.arity != 0 || d.layer != layer) continue;
        auto input = [&](uint32_t in) {
          const OpDesc& di = plan.ops[in].d;
          return di.arity ? (0x80000000u | di.arity) : di.rag_row;
        };
        plan.derive_tab.insert(plan.derive_tab.end(), {d.rag_row, input(d.a), input(d.b), d.kind == OP_CROSS ? 0u : 1u});
        ++plan.n_derive;
      }
    }
    plan.derive_tab[plan.n_layers - 1] = plan.n_derive;
    {  // the last layer's operators hold the last rows, in the table's order
      const uint32_t first = plan.derive_tab[plan.n_layers - 2], n_last = plan.n_derive - first;
      for (uint32_t i = 0; i < n_last; ++i)
        if (plan.derive_tab[hw + 4 * (first + i)] != plan.n_ragged - n_last + i) {
          err = "internal: rows of the last layer's ragged operators are out of order";
          return FBX_E_SPEC;
        }
    }
    // the crosses computed along with a multi-valued hash, grouped by hash
    const size_t n = plan.ops.size();
    uint32_t n_fused = 0;
    for (uint32_t h = 0; h < n; ++h) {
      OpDesc& dh = plan.ops[h].d;
      if (!(dh.layer == 1 && dh.kind == OP_HASH && dh.arity == 0)) continue;
      const uint32_t first = n_fused;
      for (uint32_t i : plan.nonroot_ops) {
        const OpDesc& d = plan.ops[i].d;
        if ((d.fuse == 1 && d.a == h) || (d.fuse == 2 && d.b == h)) {
          plan.derive_tab.push_back(plan.tile_lists[n + i]);
          ++n_fused;
        }
      }
      if (n_fused > 0xffffu) {
        err = "more than 65535 crosses of a multi-valued hash with a single sign";
        return FBX_E_SPEC;
      }
      dh.fuse = first | ((n_fused - first) << 16);
    }
    // Ragged operators of later layers whose count per record is scale * (count of an earlier ragged
    // operator) + add, whatever the record: a cross with a fixed-arity input, a concat with one, a concat
    // of two such operators over the same one.  Their signs before any tile follow from that operator's,
    // so the one-launch placement need not look back for them.  Three words per ragged row
    // (parent row or kNoAlias, scale, add) behind the rest of the table.
    plan.alias_at = static_cast<uint32_t>(plan.derive_tab.size());
    std::vector<uint32_t> alias(3u * plan.n_ragged, 0u);
    for (uint32_t row = 0; row < plan.n_ragged; ++row) alias[3u * row] = kNoAlias;
    for (uint32_t e = 0; e < plan.n_derive; ++e) {
      const uint32_t* d = &plan.derive_tab[hw + 4u * e];
      struct Lin { bool ok; uint32_t parent; uint64_t scale, add; };  // count = scale * count(parent) + add; parent kNoAlias: a constant
      auto lin = [&](uint32_t src) -> Lin {
        if (src >> 31) return {true, kNoAlias, 0, src & 0x7fffffffu};
        if (alias[3u * src] != kNoAlias) return {true, alias[3u * src], alias[3u * src + 1], alias[3u * src + 2]};
        return {true, src, 1, 0};
      };
      const Lin a = lin(d[1]), b = lin(d[2]);
      Lin r{false, kNoAlias, 0, 0};
      if (d[3] == 0u) {  // cross: the counts multiply
        if (a.parent == kNoAlias) r = {true, b.parent, b.scale * a.add, b.add * a.add};
        else if (b.parent == kNoAlias) r = {true, a.parent, a.scale * b.add, a.add * b.add};
      } else {           // concat: the counts add
        if (a.parent == kNoAlias || b.parent == kNoAlias || a.parent == b.parent)
          r = {true, a.parent == kNoAlias ? b.parent : a.parent, a.scale + b.scale, a.add + b.add};
      }
      if (r.ok && r.parent != kNoAlias && r.scale <= 0xffffffffull && r.add <= 0xffffffffull) {
        alias[3u * d[0]] = r.parent;
        alias[3u * d[0] + 1] = static_cast<uint32_t>(r.scale);
        alias[3u * d[0] + 2] = static_cast<uint32_t>(r.add);
        ++plan.n_alias;
      }
    }
    plan.derive_tab.insert(plan.derive_tab.end(), alias.begin(), alias.end());
  }
  return FBX_OK;
}

}  // namespace fbx
