// The "clean views" stage in toy form (Section 3 of the paper, "Clean views": null values are
// filled, fields are taken out of a JSON-like column, instances are dropped by a custom filter;
// Section 4 puts the stage on the GPU next to feature extraction).  The paper gives no algorithm
// for any of the three; the contract built here is the one stated at fbx_clean_create in
// include/fbx.h.  Output is a cleaned text buffer plus record offsets, in input order, ready to be
// handed to fbx_extract without leaving the device.
//
// Three steps on the caller's stream: every record is measured (kept or dropped, bytes of its
// cleaned form), an exclusive scan over records places the kept ones (the scan kernels of the
// extraction path), every kept record is written.
//
// Measuring and writing work on tiles of T consecutive records, the way the extraction kernel does:
// a workgroup copies the tile's text into LDS with 16-byte loads that all its lanes share, groups of
// lanes split each record at its tabs into a table of field ends (split_bytes, the extraction path's
// splitter), and lanes then are (record, field) pairs: a lane applies its field's operators, leaves
// the cleaned field's length and source in LDS, a prefix sum per record turns lengths into positions,
// and in the writing launch the lane copies its field to where it goes; neighbouring lanes write
// neighbouring fields.  A tile whose text does not fit the LDS section, and a specification with
// too many fields for the tables, take one record per thread, read in place (slow, same results).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <string>
#include <vector>

#include "fbx_device.h"
#include "fbx_split.h"

using namespace fbx;

namespace {

enum CleanKind : uint32_t { CK_FILL = 1, CK_KEY = 2, CK_KEEP = 3 };

struct CleanOp {
  uint32_t kind, field, arg_off, arg_len;
};

struct CleanParams {
  const uint8_t* raw;
  uint64_t raw_len;
  const uint64_t* rec_off;
  uint64_t n_records;
  const CleanOp* ops;         // sorted by field, spec order inside a field
  const uint32_t* first_op;   // [n_fields + 1] the operators of field k are ops[first_op[k] .. first_op[k + 1])
  const uint8_t* args;
  uint32_t n_fields;
  uint32_t* lens;             // [2][n_records]: bytes of the cleaned record (0: dropped); 1 if kept
  const uint64_t* base;       // [2][n_records]: where a kept record goes; its number among the kept ones
  const uint64_t* total;      // [2]: bytes of the output; kept records
  uint8_t* out;
  uint64_t out_cap;
  uint64_t* out_off;
  Ctrl* ctrl;
  // shape of the tile kernels (set by the host; log2T == kNoTiles: one record per thread)
  uint32_t log2T;       // records per tile
  uint32_t raw_cap;     // bytes of the text section in LDS (a multiple of 16)
  uint32_t row_stride;  // 16-bit entries per record in the table of field ends
  uint32_t o_rows, o_len, o_src;  // where the tables start in LDS
};

constexpr uint32_t kCleanThreads = 256, kCleanRawPad = 16, kCleanMaxT = 64;
constexpr uint32_t kSrcConst = 0x80000000u;  // the field's bytes come from the operators' arguments, not from the record

struct Bytes {
  const uint8_t* p;
  uint32_t n;
};

// value of the first pair "key:value" of v (pairs separated by ';') whose key is exactly name
__device__ Bytes key_value(Bytes v, const uint8_t* name, uint32_t name_len) {
  uint32_t p = 0;
  for (;;) {
    uint32_t q = p;
    while (q < v.n && v.p[q] != ';') ++q;
    uint32_t c = p;
    while (c < q && v.p[c] != ':') ++c;
    if (c < q && c - p == name_len) {
      bool same = true;
      for (uint32_t i = 0; i < name_len && same; ++i) same = v.p[p + i] == name[i];
      if (same) return Bytes{v.p + c + 1u, q - c - 1u};
    }
    if (q >= v.n) return Bytes{v.p, 0u};
    p = q + 1u;
  }
}

// Walks the F fields of one record, applies each field's operators and hands every cleaned field
// to emit(field bytes); returns false as soon as a filter drops the record.
template <class Emit>
__device__ bool clean_record(const CleanParams& C, const uint8_t* rec, uint32_t rn, Emit&& emit) {
  uint32_t p = 0;
  for (uint32_t k = 0; k < C.n_fields; ++k) {
    uint32_t q = p;
    while (q < rn && rec[q] != '\t') ++q;
    Bytes v{rec + (p <= rn ? p : rn), p <= rn ? q - p : 0u};  // (a missing field is empty)
    p = q < rn ? q + 1u : rn + 1u;
    for (uint32_t o = C.first_op[k]; o < C.first_op[k + 1]; ++o) {
      const CleanOp op = C.ops[o];
      const uint8_t* arg = C.args + op.arg_off;
      if (op.kind == CK_FILL) {
        if (v.n == 0) v = Bytes{arg, op.arg_len};
      } else if (op.kind == CK_KEY) {
        v = key_value(v, arg, op.arg_len);
      } else {
        bool ok = v.n >= op.arg_len;
        for (uint32_t i = 0; i < op.arg_len && ok; ++i) ok = v.p[i] == arg[i];
        if (!ok) return false;
      }
    }
    emit(v);
  }
  return true;
}

// the record of this thread without its trailing newline, or false (and an error bit) for bad offsets
__device__ bool clean_frame(const CleanParams& C, uint64_t r, const uint8_t*& rec, uint32_t& rn) {
  const uint64_t a = C.rec_off[r], b = C.rec_off[r + 1];
  if (a > b || b > C.raw_len) { atomicOr(&C.ctrl->err, (uint32_t)CE_OFFSETS); return false; }
  if (b - a >= (1ull << 31)) { atomicOr(&C.ctrl->err, (uint32_t)CE_TILE); return false; }
  rec = C.raw + a;
  rn = (uint32_t)(b - a);
  if (rn && rec[rn - 1u] == '\n') --rn;
  return true;
}

// ---- one record per thread, read in place
__device__ void measure_in_place(const CleanParams& C, uint64_t r) {
  const uint8_t* rec = nullptr;
  uint32_t rn = 0;
  uint64_t bytes = 0;
  bool keep = clean_frame(C, r, rec, rn);
  if (keep) keep = clean_record(C, rec, rn, [&](Bytes v) { bytes += v.n + 1ull; });  // a tab or the newline after every field
  if (keep && bytes >= (1ull << 32)) { atomicOr(&C.ctrl->err, (uint32_t)CE_TILE); keep = false; }
  C.lens[r] = keep ? (uint32_t)bytes : 0u;
  C.lens[C.n_records + r] = keep ? 1u : 0u;
}

__device__ void write_in_place(const CleanParams& C, uint64_t r) {
  if (!C.lens[C.n_records + r]) return;
  const uint8_t* rec = nullptr;
  uint32_t rn = 0;
  if (!clean_frame(C, r, rec, rn)) return;
  const uint64_t at = C.base[r];
  C.out_off[C.base[C.n_records + r]] = at;
  uint8_t* dst = C.out + at;
  uint32_t k = 0;
  clean_record(C, rec, rn, [&](Bytes v) {
    for (uint32_t i = 0; i < v.n; ++i) dst[i] = v.p[i];
    dst += v.n;
    *dst++ = ++k < C.n_fields ? '\t' : '\n';
  });
}

// What the writing launch does once: the end of the offsets array, the size the caller needs, the
// capacity check.  Returns false (in every thread of every workgroup) when nothing may be written.
__device__ bool write_may_go_ahead(const CleanParams& C, bool first_thread) {
  if (C.ctrl->err) return false;
  if (first_thread) {
    C.out_off[C.total[1]] = C.total[0];
    C.ctrl->required = C.total[0];
    if (C.total[0] > C.out_cap) atomicOr(&C.ctrl->err, (uint32_t)CE_NOMEM);
  }
  return C.total[0] <= C.out_cap;
}

__global__ __launch_bounds__(kBlock) void k_clean_measure(CleanParams C) {
  const uint64_t r = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r < C.n_records) measure_in_place(C, r);
}

__global__ __launch_bounds__(kBlock) void k_clean_write(CleanParams C) {
  const uint64_t r = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (!write_may_go_ahead(C, r == 0)) return;
  if (r < C.n_records) write_in_place(C, r);
}

// ---- tiles of records staged in LDS
extern __shared__ __align__(16) uint8_t clean_smem[];

// A cleaned field while its operators are applied: `n` bytes at position `at` of the staged text,
// or of the operators' arguments (fixed == true).
struct Field {
  uint32_t at, n;
  bool fixed;
};

// One workgroup, one tile of up to 1 << C.log2T records.  WRITE == false: the measuring launch.
template <bool WRITE>
__global__ __launch_bounds__(kCleanThreads) void k_clean_tile(CleanParams C) {
  __shared__ uint64_t s_off[kCleanMaxT + 1];
  __shared__ uint64_t s_base[kCleanMaxT];
  __shared__ uint32_t s_rs[kCleanMaxT], s_re[kCleanMaxT], s_len[kCleanMaxT], s_drop[kCleanMaxT];
  __shared__ uint32_t s_bad;
  __shared__ uint32_t s_go;
  const uint32_t tid = threadIdx.x;
  if (WRITE) {  // (one thread decides for the workgroup: the error word may change while the launch runs)
    if (tid == 0) s_go = write_may_go_ahead(C, blockIdx.x == 0) ? 1u : 0u;
    __syncthreads();
    if (!s_go) return;
  }
  const uint32_t T = 1u << C.log2T, F = C.n_fields;
  const uint64_t g0 = (uint64_t)blockIdx.x << C.log2T;
  if (g0 >= C.n_records) return;  // (an empty batch still launches one workgroup, for the lines above)
  const uint32_t nb = (uint32_t)min((uint64_t)T, C.n_records - g0);
  uint8_t* raw = clean_smem;
  uint16_t* rows = reinterpret_cast<uint16_t*>(clean_smem + C.o_rows);
  uint32_t* flen = reinterpret_cast<uint32_t*>(clean_smem + C.o_len);  // bytes of the cleaned field and its separator, then where it starts in the cleaned record
  uint32_t* fsrc = reinterpret_cast<uint32_t*>(clean_smem + C.o_src);  // where its bytes come from
  if (tid == 0) s_bad = 0;
  if (tid <= nb) s_off[tid] = C.rec_off[g0 + tid];
  if (tid < kCleanMaxT) s_drop[tid] = 0;
  __syncthreads();
  if (tid < nb) {
    const uint64_t a = s_off[tid], b = s_off[tid + 1];
    if (a > b || b > C.raw_len) atomicOr(&s_bad, (uint32_t)CE_OFFSETS);
    else if (b - a >= (1ull << 31)) atomicOr(&s_bad, (uint32_t)CE_TILE);
  }
  __syncthreads();
  if (s_bad) {  // the call fails; the arrays the scan reads still get defined values
    if (tid == 0) atomicOr(&C.ctrl->err, s_bad);
    if (!WRITE && tid < nb) C.lens[g0 + tid] = C.lens[C.n_records + g0 + tid] = 0u;
    return;
  }
  const uint64_t o0 = s_off[0];
  const uintptr_t ok_lo = reinterpret_cast<uintptr_t>(C.raw), ok_hi = ok_lo + C.raw_len;
  const uint32_t delta = (uint32_t)((ok_lo + o0) & 15u);
  if (s_off[nb] - o0 + delta > (uint64_t)C.raw_cap) {  // the text does not fit the section
    if (tid < nb) {
      if (WRITE) write_in_place(C, g0 + tid); else measure_in_place(C, g0 + tid);
    }
    return;
  }
  {  // the tile's text, in whole 16-byte chunks
    const uint32_t nchunks = (delta + (uint32_t)(s_off[nb] - o0) + 15u) >> 4;
    const uintptr_t a0 = ok_lo + o0 - delta;
    for (uint32_t c = tid; c < nchunks; c += kCleanThreads) {
      const uintptr_t ca = a0 + 16u * c;
      u32x4 v;
      if (ca >= ok_lo && ca + 16u <= ok_hi) {
        v = *reinterpret_cast<const u32x4*>(ca);
      } else {  // a chunk across an end of the caller's buffer: what lies outside reads as zero
        uint32_t w[4] = {0, 0, 0, 0};
        for (uint32_t i = 0; i < 16; ++i) {
          const uintptr_t bi = ca + i;
          if (bi >= ok_lo && bi < ok_hi) w[i >> 2] |= (uint32_t)*reinterpret_cast<const uint8_t*>(bi) << (8u * (i & 3u));
        }
        v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
      }
      *reinterpret_cast<u32x4*>(raw + kCleanRawPad + 16u * c) = v;
    }
    if (tid < nb) {
      s_rs[tid] = kCleanRawPad + delta + (uint32_t)(s_off[tid] - o0);
      s_re[tid] = kCleanRawPad + delta + (uint32_t)(s_off[tid + 1] - o0);
    }
  }
  __syncthreads();
  // field ends: 256 / T lanes (at most 64) share a record; entries from the record's tab count on hold its end
  const uint32_t lg = 8u - C.log2T < 6u ? 8u - C.log2T : 6u;
  const uint32_t gsz = 1u << lg, j = tid & (gsz - 1u), rr = tid >> lg;
  const bool act = rr < nb;
  uint32_t rs = 0, re = 0;
  if (act) {
    rs = s_rs[rr]; re = s_re[rr];
    if (re > rs && raw[re - 1u] == '\n') --re;  // one trailing newline is not part of the record
  }
  uint16_t* row = rows + rr * C.row_stride;
  {
    const uint32_t tabs = split_bytes(raw, rs, re, act, kTabs, lg, j, F, [&](uint32_t k, uint32_t pos) { row[1u + k] = (uint16_t)pos; });
    if (act) {
      if (j == 0) row[0] = (uint16_t)(rs - 1u);
      for (uint32_t kk = tabs + j; kk < F; kk += gsz) row[1u + kk] = (uint16_t)re;
    }
  }
  __syncthreads();
  // lanes as (record, field) pairs: a wavefront takes a record, its lanes the fields
  auto byte_of = [&](const Field& f, uint32_t i) -> uint32_t { return f.fixed ? C.args[f.at + i] : raw[f.at + i]; };
  for (uint32_t r = tid >> 6; r < nb; r += kCleanThreads / 64u) {
    const uint16_t* rw = rows + r * C.row_stride;
    for (uint32_t k = tid & 63u; k < F; k += 64u) {
      const uint32_t s = (uint32_t)rw[k] + 1u, e = rw[k + 1u];
      Field f{s, e > s ? e - s : 0u, false};  // (a missing field is empty)
      bool keep = true;
      for (uint32_t o = C.first_op[k]; o < C.first_op[k + 1] && keep; ++o) {
        const CleanOp op = C.ops[o];
        if (op.kind == CK_FILL) {
          if (f.n == 0) f = Field{op.arg_off, op.arg_len, true};
        } else if (op.kind == CK_KEY) {
          // value of the first pair "key:value" (pairs separated by ';') whose key is exactly the name
          uint32_t p = 0;
          for (;;) {
            uint32_t q = p;
            while (q < f.n && byte_of(f, q) != ';') ++q;
            uint32_t c = p;
            while (c < q && byte_of(f, c) != ':') ++c;
            if (c < q && c - p == op.arg_len) {
              bool same = true;
              for (uint32_t i = 0; i < op.arg_len && same; ++i) same = byte_of(f, p + i) == C.args[op.arg_off + i];
              if (same) { f.at += c + 1u; f.n = q - c - 1u; break; }
            }
            if (q >= f.n) { f.n = 0; break; }
            p = q + 1u;
          }
        } else {
          keep = f.n >= op.arg_len;
          for (uint32_t i = 0; i < op.arg_len && keep; ++i) keep = byte_of(f, i) == C.args[op.arg_off + i];
        }
      }
      if (!keep) s_drop[r] = 1u;
      flen[r * F + k] = f.n + 1u;  // a tab or the newline after every field
      fsrc[r * F + k] = f.at | (f.fixed ? kSrcConst : 0u);
    }
  }
  __syncthreads();
  {  // lengths become positions inside the cleaned record: the lanes that shared the record's tabs share its fields
    const uint32_t c = (F + gsz - 1u) >> lg;
    const uint32_t k0 = min(j * c, F), k1 = min(k0 + c, F);
    uint32_t sum = 0;
    if (act) for (uint32_t k = k0; k < k1; ++k) sum += flen[rr * F + k];
    const uint32_t incl = group_prefix(sum, lg, j);
    const uint32_t total = __shfl(incl, (int)(lane_id() | (gsz - 1u)), 64);
    if (act) {
      uint32_t at = incl - sum;
      for (uint32_t k = k0; k < k1; ++k) {
        const uint32_t n = flen[rr * F + k];
        flen[rr * F + k] = at;
        at += n;
      }
      if (j == 0) s_len[rr] = total;
    }
  }
  __syncthreads();
  if (!WRITE) {
    if (tid < nb) {
      const bool kept = !s_drop[tid];
      C.lens[g0 + tid] = kept ? s_len[tid] : 0u;
      C.lens[C.n_records + g0 + tid] = kept ? 1u : 0u;
    }
    return;
  }
  if (tid < nb && !s_drop[tid]) {
    const uint64_t at = C.base[g0 + tid];
    s_base[tid] = at;
    C.out_off[C.base[C.n_records + g0 + tid]] = at;
  }
  __syncthreads();
  for (uint32_t r = tid >> 6; r < nb; r += kCleanThreads / 64u) {
    if (s_drop[r]) continue;
    for (uint32_t k = tid & 63u; k < F; k += 64u) {
      const uint32_t at = flen[r * F + k];
      const uint32_t n = (k + 1u < F ? flen[r * F + k + 1u] : s_len[r]) - at - 1u;
      const uint32_t src = fsrc[r * F + k];
      uint8_t* dst = C.out + s_base[r] + at;
      if (src & kSrcConst) {
        const uint8_t* from = C.args + (src & ~kSrcConst);
        for (uint32_t i = 0; i < n; ++i) dst[i] = from[i];
      } else {
        const uint8_t* from = raw + src;
        for (uint32_t i = 0; i < n; ++i) dst[i] = from[i];
      }
      dst[n] = k + 1u < F ? '\t' : '\n';
    }
  }
}

uint64_t up256(uint64_t x) { return (x + 255u) & ~uint64_t(255); }

int hex_digit(char c) {
  if (c >= '0' && c <= '9') return c - '0';
  if (c >= 'a' && c <= 'f') return c - 'a' + 10;
  if (c >= 'A' && c <= 'F') return c - 'A' + 10;
  return -1;
}

thread_local std::string g_clean_create_error;

}  // namespace

struct fbx_clean {
  uint32_t n_fields = 0;
  std::vector<CleanOp> ops;          // sorted by field (stable)
  std::vector<uint32_t> first_op;    // n_fields + 1
  std::vector<uint8_t> args;
  std::vector<uint8_t> image;        // ops, first_op, args as they lie in the scratch
  uint64_t off_ops = 0, off_first = 0, off_args = 0, off_tables_end = 0;
  std::string error;
};

namespace {

struct CleanLayout {
  uint64_t ctrl, total, tables, lens, base, part, end;
};

CleanLayout clean_layout(const fbx_clean& c, uint64_t n) {
  CleanLayout L{};
  uint64_t o = 0;
  L.ctrl = o; o = up256(o + sizeof(Ctrl));
  L.total = o; o = up256(o + 16);
  L.tables = o; o = up256(o + c.image.size());
  L.lens = o; o = up256(o + 2 * n * 4);
  L.base = o; o = up256(o + 2 * n * 8);
  L.part = o; o = up256(o + 2ull * scan_segments(static_cast<uint32_t>(n)) * 8);
  L.end = o;
  return L;
}

}  // namespace

extern "C" {

fbx_status fbx_clean_create(const char* spec, size_t spec_len, fbx_clean** out) {
  if (!spec || !out) { g_clean_create_error = "spec and out must not be NULL"; return FBX_E_ARG; }
  std::unique_ptr<fbx_clean> c(new (std::nothrow) fbx_clean());
  if (!c) return FBX_E_ARG;
  std::vector<CleanOp> in_spec_order;
  const std::string text(spec, spec_len);
  size_t pos = 0;
  int line_no = 0;
  bool header = false;
  auto fail = [&](const std::string& why) {
    g_clean_create_error = "line " + std::to_string(line_no) + ": " + why;
    return FBX_E_SPEC;
  };
  while (pos <= text.size()) {
    size_t nl = text.find('\n', pos);
    if (nl == std::string::npos) nl = text.size();
    std::string line = text.substr(pos, nl - pos);
    pos = nl + 1;
    ++line_no;
    const size_t hash = line.find('#');
    if (hash != std::string::npos) line.resize(hash);
    std::vector<std::string> words;
    for (size_t i = 0; i < line.size();) {
      while (i < line.size() && (line[i] == ' ' || line[i] == '\t' || line[i] == '\r')) ++i;
      size_t j = i;
      while (j < line.size() && line[j] != ' ' && line[j] != '\t' && line[j] != '\r') ++j;
      if (j > i) words.push_back(line.substr(i, j - i));
      i = j;
    }
    if (words.empty()) continue;
    if (!header) {
      if (words.size() != 2 || words[0] != "fbxclean" || words[1] != "1") return fail("expected 'fbxclean 1'");
      header = true;
      continue;
    }
    if (words[0] == "fields") {
      char* end = nullptr;
      const unsigned long f = words.size() == 2 ? strtoul(words[1].c_str(), &end, 10) : 0;
      if (words.size() != 2 || *end || f == 0 || f > 65535 || c->n_fields) return fail("bad or repeated 'fields'");
      c->n_fields = static_cast<uint32_t>(f);
      continue;
    }
    CleanOp op{};
    const char* arg_key = nullptr;
    if (words[0] == "fill") { op.kind = CK_FILL; arg_key = "value"; }
    else if (words[0] == "key") { op.kind = CK_KEY; arg_key = "name"; }
    else if (words[0] == "keep") { op.kind = CK_KEEP; arg_key = "prefix"; }
    if (!op.kind || !c->n_fields) return fail("unknown operator, or an operator before 'fields'");
    bool have_field = false, have_arg = false;
    for (size_t w = 1; w < words.size(); ++w) {
      const size_t eq = words[w].find('=');
      if (eq == std::string::npos) return fail("expected key=value");
      const std::string key = words[w].substr(0, eq), val = words[w].substr(eq + 1);
      if (key == "field" && !have_field) {
        char* end = nullptr;
        const unsigned long f = strtoul(val.c_str(), &end, 10);
        if (val.empty() || *end || f >= c->n_fields) return fail("field out of range");
        op.field = static_cast<uint32_t>(f);
        have_field = true;
      } else if (key == arg_key && !have_arg) {
        if (val.size() % 2 || val.size() / 2 > 255) return fail("bytes are written as an even number of hex digits, at most 255 bytes");
        op.arg_off = static_cast<uint32_t>(c->args.size());
        op.arg_len = static_cast<uint32_t>(val.size() / 2);
        for (size_t i = 0; i < val.size(); i += 2) {
          const int hi = hex_digit(val[i]), lo = hex_digit(val[i + 1]);
          if (hi < 0 || lo < 0) return fail("bad hex digit");
          const uint8_t b = static_cast<uint8_t>(hi * 16 + lo);
          if (op.kind == CK_FILL && (b == '\t' || b == '\n')) return fail("a fill value holds no tab and no newline");
          c->args.push_back(b);
        }
        have_arg = true;
      } else {
        return fail("unknown or repeated key '" + key + "'");
      }
    }
    if (!have_field || !have_arg) return fail("missing key");
    if (op.kind == CK_FILL && op.arg_len == 0) return fail("a fill value is not empty");
    in_spec_order.push_back(op);
  }
  if (!header || !c->n_fields) { ++line_no; return fail("missing header or 'fields'"); }
  c->ops = in_spec_order;
  std::stable_sort(c->ops.begin(), c->ops.end(), [](const CleanOp& a, const CleanOp& b) { return a.field < b.field; });
  c->first_op.assign(c->n_fields + 1, 0);
  for (const CleanOp& op : c->ops) ++c->first_op[op.field + 1];
  for (uint32_t k = 0; k < c->n_fields; ++k) c->first_op[k + 1] += c->first_op[k];
  uint64_t o = 0;
  c->off_ops = o; o = up256(o + c->ops.size() * sizeof(CleanOp));
  c->off_first = o; o = up256(o + c->first_op.size() * 4);
  c->off_args = o; o = up256(o + c->args.size());
  c->image.assign(o, 0);
  if (!c->ops.empty()) std::memcpy(c->image.data() + c->off_ops, c->ops.data(), c->ops.size() * sizeof(CleanOp));
  std::memcpy(c->image.data() + c->off_first, c->first_op.data(), c->first_op.size() * 4);
  if (!c->args.empty()) std::memcpy(c->image.data() + c->off_args, c->args.data(), c->args.size());
  *out = c.release();
  return FBX_OK;
}

void fbx_clean_destroy(fbx_clean* clean) { delete clean; }

const char* fbx_clean_last_error(const fbx_clean* clean) { return clean ? clean->error.c_str() : g_clean_create_error.c_str(); }

fbx_status fbx_clean_scratch_hint(const fbx_clean* clean, uint64_t n_records, uint64_t* bytes) {
  if (!clean || !bytes || n_records >= (1ull << 32)) return FBX_E_ARG;
  *bytes = clean_layout(*clean, n_records).end;
  return FBX_OK;
}

fbx_status fbx_clean_run(fbx_clean* clean, const uint8_t* d_raw, uint64_t raw_len, const uint64_t* d_rec_off,
                         uint64_t n_records, uint8_t* d_out, uint64_t out_cap, uint64_t* d_out_off, void* d_scratch,
                         uint64_t scratch_bytes, void* hip_stream, fbx_clean_result* out) {
  if (!clean || !out || !d_rec_off || (!d_raw && raw_len) || !d_out_off || (!d_out && out_cap) || !d_scratch) {
    if (clean) clean->error = "NULL argument";
    return FBX_E_ARG;
  }
  if (n_records >= (1ull << 32) || (reinterpret_cast<uintptr_t>(d_scratch) & 255u)) {
    clean->error = "a call takes fewer than 2^32 records and a 256-byte aligned scratch buffer";
    return FBX_E_ARG;
  }
  const CleanLayout L = clean_layout(*clean, n_records);
  out->n_kept = out->out_len = 0;
  out->required_scratch = L.end;
  if (scratch_bytes < L.end) {
    clean->error = "scratch buffer too small: need " + std::to_string(L.end) + " bytes";
    return FBX_E_NOMEM;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* sc = static_cast<uint8_t*>(d_scratch);
  auto hip_failed = [&](hipError_t e, const char* where) {
    clean->error = std::string(where) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    return FBX_E_HIP;
  };
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(sc + L.ctrl);
  uint64_t* total = reinterpret_cast<uint64_t*>(sc + L.total);
  hipError_t e = launch_reset(ctrl, 0, st);
  if (e == hipSuccess) e = launch_fill64(total, 2, 0, st);
  if (e == hipSuccess) e = hipMemcpyAsync(sc + L.tables, clean->image.data(), clean->image.size(), hipMemcpyHostToDevice, st);
  if (e != hipSuccess) return hip_failed(e, "set-up");
  CleanParams C{};
  C.raw = d_raw; C.raw_len = raw_len; C.rec_off = d_rec_off; C.n_records = n_records;
  C.ops = reinterpret_cast<const CleanOp*>(sc + L.tables + clean->off_ops);
  C.first_op = reinterpret_cast<const uint32_t*>(sc + L.tables + clean->off_first);
  C.args = sc + L.tables + clean->off_args;
  C.n_fields = clean->n_fields;
  C.lens = reinterpret_cast<uint32_t*>(sc + L.lens);
  C.base = reinterpret_cast<const uint64_t*>(sc + L.base);
  C.total = total;
  C.out = d_out; C.out_cap = out_cap; C.out_off = d_out_off; C.ctrl = ctrl;
  // Tiles: as many records as usually fit the text section with room to spare, their tables within the
  // budget; the three sections stay under the 64 KiB a workgroup gets without asking for more.
  constexpr uint32_t kTextMax = 24576, kTableMax = 32768;
  const uint64_t mean = n_records ? raw_len / n_records + 1 : 1;
  const uint64_t F = clean->n_fields;
  const uint64_t row_stride = (F + 2 + 7) & ~uint64_t(7);
  auto tables = [&](uint64_t T) { return T * (row_stride * 2 + F * 8); };
  uint32_t log2T = 6;
  while (log2T && ((mean << log2T) * 5 / 4 > kTextMax || tables(1ull << log2T) > kTableMax)) --log2T;
  const bool tiles = tables(1ull << log2T) <= kTableMax;
  uint32_t lds = 0;
  if (tiles) {
    const uint64_t T = 1ull << log2T;
    C.log2T = log2T;
    C.raw_cap = static_cast<uint32_t>(std::min<uint64_t>(kTextMax, std::max<uint64_t>(4096, (T * mean * 3 / 2 + 64 + 15) & ~uint64_t(15))));
    C.row_stride = static_cast<uint32_t>(row_stride);
    C.o_rows = kCleanRawPad + C.raw_cap + 16;  // (the splitter reads whole 16-byte chunks: one more behind the text)
    C.o_len = static_cast<uint32_t>(C.o_rows + T * row_stride * 2);
    C.o_src = static_cast<uint32_t>(C.o_len + T * F * 4);
    lds = static_cast<uint32_t>(C.o_src + T * F * 4);
  }
  const uint32_t blocks = tiles ? static_cast<uint32_t>((n_records + (1ull << log2T) - 1) >> log2T)
                                : static_cast<uint32_t>((n_records + kBlock - 1) / kBlock);
  if (n_records) {
    if (tiles) hipLaunchKernelGGL(k_clean_tile<false>, dim3(blocks), dim3(kCleanThreads), lds, st, C);
    else hipLaunchKernelGGL(k_clean_measure, dim3(blocks), dim3(kBlock), 0, st, C);
    e = hipGetLastError();
    if (e == hipSuccess)
      e = launch_scan(C.lens, reinterpret_cast<uint64_t*>(sc + L.base), total, reinterpret_cast<uint64_t*>(sc + L.part), 2,
                      static_cast<uint32_t>(n_records), ctrl, st);
    if (e != hipSuccess) return hip_failed(e, "measuring and placing records");
  }
  if (tiles) hipLaunchKernelGGL(k_clean_tile<true>, dim3(std::max(blocks, 1u)), dim3(kCleanThreads), lds, st, C);
  else hipLaunchKernelGGL(k_clean_write, dim3(std::max(blocks, 1u)), dim3(kBlock), 0, st, C);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_failed(e, "writing records");
  struct { Ctrl c; uint8_t pad[256 - sizeof(Ctrl)]; uint64_t total[2]; } back;
  static_assert(sizeof(back) == 256 + 16, "read-back layout");
  e = hipMemcpyAsync(&back, sc + L.ctrl, sizeof back, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_failed(e, "read-back");
  if (back.c.err & CE_OFFSETS) { clean->error = "record offsets must be non-decreasing and end within raw_len"; return FBX_E_INPUT; }
  if (back.c.err & CE_TILE) { clean->error = "a record of 2 GiB or more, or one that cleans to 4 GiB or more"; return FBX_E_INPUT; }
  out->n_kept = back.total[1];
  out->out_len = back.total[0];
  if (back.c.err & CE_NOMEM) {
    clean->error = "output buffer too small: need " + std::to_string(back.total[0]) + " bytes";
    return FBX_E_NOMEM;
  }
  clean->error.clear();
  return FBX_OK;
}

}  // extern "C"
