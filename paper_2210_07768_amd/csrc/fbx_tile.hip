// The tile kernel of libfbx for gfx950 (MI355X).
//
// Work decomposition.  Records are independent (every operator computes on one
// row of the table; Section 3, "Extract features"), so a workgroup owns a tile
// of T consecutive records (T a power of two, at most 64) and takes it through
// every layer of the operator graph in order (Section 4, "Scheduling"): the
// synchronisation after a layer is a workgroup barrier, because no record ever
// reads another record's signs.
//
//  1. The tile's raw text, one contiguous byte range, is copied into LDS with
//     16-byte loads that every lane of the workgroup takes part in: each raw
//     byte leaves HBM once, fully coalesced.
//  2. Splitting at the delimiter (Section 5, first paragraph): groups of lanes
//     share a record, find its tabs four bytes at a time and write a table of
//     field ends (16-bit LDS positions).  No per-thread array is allocated; the
//     table has one entry per (record, field).
//  3. Layer 1: lanes are (record, operator) pairs.  A lane looks up its field in
//     the table and hashes / parses it out of LDS; T neighbouring lanes hold T
//     consecutive records of one operator, so a slot is written in runs of 8 T
//     bytes.  Signs that a later operator needs stay in an LDS table as well.
//  4. Later layers read their inputs from that table (or, for lists, from the
//     arrays this workgroup wrote) after the barrier.
//  5. Ragged slots: the per-record counts of the tile are found first, then
//     turned into positions by a prefix sum over the tile's records on top of
//     the tile's base (a counting launch of this same kernel and a scan over
//     tiles provide it).
//
// A tile whose text does not fit the LDS section is worked off in several
// passes of fewer records; a single record that does not fit alone is walked
// straight from memory, one lane per operator (slow, rare, same results).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "fbx_device.h"

namespace fbx {
namespace {

constexpr uint32_t kNoRow = 0xffffffffu;
constexpr uint64_t kPrime = 0x100000001b3ull;
constexpr uint32_t kMaxCount = 0x3ffffffu;  // signs per record and operator

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

extern __shared__ __align__(16) uint8_t smem[];

// Phase timing for tuning builds (-DFBX_TILE_PROF): wavefront 0 charges the cycles
// since its last mark to a phase; the sums of all workgroups land in P.prof.
#ifdef FBX_TILE_PROF
__shared__ unsigned long long s_prof[16];
__shared__ unsigned long long s_prof_last;
#define FBX_MARK(n)                                             \
  do {                                                          \
    if (threadIdx.x == 0) {                                     \
      const unsigned long long now_ = clock64();                \
      s_prof[n] += now_ - s_prof_last;                          \
      s_prof_last = now_;                                       \
    }                                                           \
  } while (0)
#else
#define FBX_MARK(n) do {} while (0)
#endif

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

// Views of the LDS sections of one workgroup.
struct Sh {
  uint64_t* off;    // [T + 1] record offsets of the tile
  uint32_t* rs;     // [T] LDS position of the first byte of a staged record
  uint32_t* re;     // [T] LDS position one past its last byte (newline dropped)
  uint16_t* rows;   // [T][row_stride]: row[0] = rs - 1, row[1 + k] = end of field k
  uint8_t* raw;     // staged text; byte 0 of the staged range sits at kRawPad + (address & 15)
  uint64_t* stage;  // [n_stage][T] single signs kept for later layers
  uint32_t* cnt;    // [n_ragged][T] signs of a ragged operator per record
  uint32_t* start;  // [n_ragged][T] their first position, relative to the tile's base
  uint32_t* run;    // [n_ragged] signs of the tile's earlier passes
  uint64_t* base;   // [n_ragged] the tile's base in the operator's values array
  // plan tables, copied once per workgroup so that no lane waits on memory for a descriptor
  const OpProg* prog;          // [n_ops]
  const uint32_t* lists;       // work lists (operator indices)
  const uint32_t* list_begin;
  const uint32_t* rnr;         // ragged operators of layers >= 2, spec order
  const uint8_t* aux;          // bucket boundaries and filter prefixes
};

__device__ __forceinline__ Sh views(const TileParams& P) {
  Sh s;
  s.off = reinterpret_cast<uint64_t*>(smem + P.o_off);
  s.rs = reinterpret_cast<uint32_t*>(smem + P.o_rs);
  s.re = reinterpret_cast<uint32_t*>(smem + P.o_re);
  s.rows = reinterpret_cast<uint16_t*>(smem + P.o_rows);
  s.raw = smem + P.o_raw;
  s.stage = reinterpret_cast<uint64_t*>(smem + P.o_stage);
  s.cnt = reinterpret_cast<uint32_t*>(smem + P.o_cnt);
  s.start = reinterpret_cast<uint32_t*>(smem + P.o_start);
  s.run = reinterpret_cast<uint32_t*>(smem + P.o_run);
  s.base = reinterpret_cast<uint64_t*>(smem + P.o_base);
  s.prog = reinterpret_cast<const OpProg*>(smem + P.o_prog);
  s.lists = reinterpret_cast<const uint32_t*>(smem + P.o_lists);
  s.list_begin = reinterpret_cast<const uint32_t*>(smem + P.o_lbeg);
  s.rnr = reinterpret_cast<const uint32_t*>(smem + P.o_rnr);
  s.aux = smem + P.o_aux;
  return s;
}

// ------------------------------------------------------------ byte sources
// Where a lane reads record bytes from.  Positions are 32-bit.
struct LdsSrc {
  const uint8_t* raw8;
  const uint16_t* rows;
  uint32_t stride;
  __device__ __forceinline__ uint32_t byte(uint32_t p) const { return raw8[p]; }
  // Field k of staged record r: [s, e).  A missing field is empty.
  __device__ __forceinline__ void span(uint32_t r, uint32_t k, uint32_t& s, uint32_t& e) const {
    const uint16_t* row = rows + r * stride + k;
    s = (uint32_t)row[0] + 1u;
    e = row[1];
    if (e < s) e = s;
  }
};

// One record read in place (it does not fit the LDS section); positions count from its first byte.
struct GlobalSrc {
  const uint8_t* rec;
  uint32_t len;  // newline dropped
  __device__ __forceinline__ uint32_t byte(uint32_t p) const { return rec[p]; }
  __device__ __forceinline__ void span(uint32_t, uint32_t k, uint32_t& s, uint32_t& e) const {
    uint32_t p = 0, f = 0;
    while (f < k && p < len) {
      if (rec[p] == '\t') ++f;
      ++p;
    }
    if (f < k) { s = e = len; return; }
    s = p;
    while (p < len && rec[p] != '\t') ++p;
    e = p;
  }
};

// ------------------------------------------------------------ splitting
// 0x80 in exactly the bytes of w that are tabs.
__device__ __forceinline__ uint32_t tab_flags(uint32_t w) {
  const uint32_t x = w ^ 0x09090909u;
  return ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);
}

// Field table of the staged records.  kTileThreads / T lanes (at most 64) share a
// record: each takes an equal run of its dwords, counts its tabs, a prefix sum
// over the group turns the counts into field numbers, and a second walk writes
// the positions.  Entries from the record's tab count on hold the record's end.
__device__ void tokenize(const TileParams& P, const Sh& sh, uint32_t nb) {
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t kLogThreads = kTileThreads == 1024 ? 10u : (kTileThreads == 512 ? 9u : 8u);
  const uint32_t lg = kLogThreads - P.log2T < 6u ? kLogThreads - P.log2T : 6u;  // log2 of the lanes per record
  const uint32_t gsz = 1u << lg;
  const uint32_t j = tid & (gsz - 1u);
  const uint32_t r = tid >> lg;
  const uint32_t F = P.n_fields;
  const bool act = r < nb;
  uint32_t rs = 0, re = 0;
  if (act) { rs = sh.rs[r]; re = sh.re[r]; }
  const uint32_t ab = rs & ~3u;
  const uint32_t nd = (act && re > rs) ? (re - ab + 3u) >> 2 : 0u;  // dwords that cover the record
  const uint32_t c = (nd + gsz - 1u) >> lg;                         // dwords per lane
  const uint32_t d0 = min(j * c, nd), d1 = min(d0 + c, nd);
  const uint32_t* raw32 = reinterpret_cast<const uint32_t*>(sh.raw);
  auto flags_at = [&](uint32_t d) {
    uint32_t f = tab_flags(raw32[(ab >> 2) + d]);
    if (d == 0) f &= 0xffffffffu << ((rs & 3u) * 8u);  // bytes before the record
    const uint32_t rem = re - (ab + 4u * d);           // bytes of the record from this dword on (>= 1)
    if (rem < 4u) f &= (1u << (rem * 8u)) - 1u;        // bytes after the record
    return f;
  };
  uint32_t cnt = 0;
  for (uint32_t d = d0; d < d1; ++d) cnt += __popc(flags_at(d));
  uint32_t incl = cnt;
  for (uint32_t s = 1; s < gsz; s <<= 1) {
    const uint32_t t = __shfl_up(incl, s, 64);
    if (j >= s) incl += t;
  }
  const uint32_t total = __shfl(incl, (int)(lane_id() | (gsz - 1u)), 64);
  if (!act) return;
  uint32_t k = incl - cnt;
  uint16_t* row = sh.rows + r * P.row_stride;
  for (uint32_t d = d0; d < d1; ++d) {
    uint32_t f = flags_at(d);
    while (f) {
      const uint32_t b = (uint32_t)__ffs((int)f) - 1u;  // 7, 15, 23 or 31
      if (k < F) row[1u + k] = (uint16_t)(ab + 4u * d + (b >> 3));
      ++k;
      f &= f - 1u;
    }
  }
  if (j == 0) row[0] = (uint16_t)(rs - 1u);
  for (uint32_t kk = total + j; kk < F; kk += gsz) row[1u + kk] = (uint16_t)re;
}

// ------------------------------------------------------------ token operators
// Eight staged bytes starting at position p (any alignment), in two dwords.
__device__ __forceinline__ void window8(const LdsSrc& src, uint32_t p, uint32_t& x0, uint32_t& x1) {
  const uint32_t* raw32 = reinterpret_cast<const uint32_t*>(src.raw8);
  const uint32_t a = p >> 2, sh = (p & 3u) * 8u;
  const uint32_t w0 = raw32[a], w1 = raw32[a + 1], w2 = raw32[a + 2];
  x0 = __builtin_amdgcn_alignbit(w1, w0, sh);
  x1 = __builtin_amdgcn_alignbit(w2, w1, sh);
}

// Calls f(byte) for every byte of [s, e), in order.  Staged text is read eight
// bytes per window; the steps of a window nest, so a lane that is done leaves
// the execution mask once.
template <class F>
__device__ __forceinline__ void for_each_byte(const LdsSrc& src, uint32_t s, uint32_t e, F&& f) {
  uint32_t p = s;
  while (p < e) {
    uint32_t x0, x1;
    window8(src, p, x0, x1);
    const uint32_t n = e - p < 8u ? e - p : 8u;
#define FBX_STEP(J, X) if (n > (uint32_t)J) { f(((X) >> (8 * (J & 3))) & 0xffu);
    FBX_STEP(0, x0) FBX_STEP(1, x0) FBX_STEP(2, x0) FBX_STEP(3, x0)
    FBX_STEP(4, x1) FBX_STEP(5, x1) FBX_STEP(6, x1) FBX_STEP(7, x1)
    }}}}}}}}
#undef FBX_STEP
    p += n;
  }
}

template <class F>
__device__ __forceinline__ void for_each_byte(const GlobalSrc& src, uint32_t s, uint32_t e, F&& f) {
  for (uint32_t p = s; p < e; ++p) f(src.byte(p));
}

// FNV-1a over the bytes [s, e) from state h.
template <class Src>
__device__ __forceinline__ uint64_t hash_span(const Src& src, uint32_t s, uint32_t e, uint64_t h) {
  for_each_byte(src, s, e, [&](uint32_t b) { h = (h ^ b) * kPrime; });
  return h;
}

// 0x80 in exactly the zero bytes of x.
__device__ __forceinline__ uint32_t zero_exact(uint32_t x) {
  return ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);
}

// Number of commas in [s, e).
__device__ __forceinline__ uint32_t count_commas(const LdsSrc& src, uint32_t s, uint32_t e) {
  uint32_t c = 0;
  for (uint32_t p = s; p < e; p += 8u) {
    uint32_t x0, x1;
    window8(src, p, x0, x1);
    const uint32_t n = e - p;  // bytes left, >= 1
    uint32_t f0 = zero_exact(x0 ^ 0x2c2c2c2cu), f1 = zero_exact(x1 ^ 0x2c2c2c2cu);
    if (n < 4u) f0 &= (1u << (8u * n)) - 1u;
    if (n <= 4u) f1 = 0;
    else if (n < 8u) f1 &= (1u << (8u * (n - 4u))) - 1u;
    c += __popc(f0) + __popc(f1);
  }
  return c;
}

__device__ __forceinline__ uint32_t count_commas(const GlobalSrc& src, uint32_t s, uint32_t e) {
  uint32_t c = 0;
  for (uint32_t p = s; p < e; ++p) c += src.byte(p) == ',' ? 1u : 0u;
  return c;
}

struct NumState {
  uint64_t ip = 0, fp = 0;
  uint32_t digits = 0, nfrac = 0, st = 0;  // st: 0 start, 1 integer part, 2 fraction, 3 stopped early
  bool neg = false;
  __device__ __forceinline__ void step(uint32_t b) {
    if (st == 3) return;
    if (st == 0) {
      st = 1;
      if (b == '-') { neg = true; return; }
    }
    const uint32_t d = b - '0';
    if (st == 1) {
      if (d <= 9) { ip = ip * 10u + d; ++digits; }
      else if (b == '.') st = 2;
      else st = 3;
    } else {
      if (d <= 9) {
        if (nfrac < 6) { fp = fp * 10u + d; ++nfrac; }
        ++digits;
      } else st = 3;
    }
  }
  // signed micro-units; bad when the text was not wholly -?digits*(.digits*)? with a digit
  __device__ __forceinline__ int64_t finish(bool& bad) {
    for (; nfrac < 6; ++nfrac) fp *= 10u;
    uint64_t v = ip * 1000000ull + fp;
    if (neg) v = 0ull - v;
    bad = st == 3 || digits == 0;
    return (int64_t)v;
  }
};

__device__ __forceinline__ uint64_t bucket_sign(const OpProg& d, const uint8_t* aux, NumState& ns, uint32_t& malformed) {
  bool bad;
  const int64_t v = ns.finish(bad);
  malformed += bad ? 1u : 0u;
  const int64_t* b = reinterpret_cast<const int64_t*>(aux + d.aux_off);
  uint32_t lo = 0, hi = d.aux_len;  // index = number of boundaries <= v
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (b[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return mix64(d.key + lo);
}

// The one sign of a single-valued hash or bucket operator on [s, e).
template <class Src>
__device__ __forceinline__ uint64_t single_sign(const Src& src, const OpProg& d, const uint8_t* aux, uint32_t s,
                                                uint32_t e, uint32_t& malformed) {
  if (d.kind == OP_HASH) return hash_span(src, s, e, d.key);
  NumState ns;
  for_each_byte(src, s, e, [&](uint32_t b) { ns.step(b); });
  return bucket_sign(d, aux, ns, malformed);
}

// Number of signs a ragged root operator (not n-gram) produces on [s, e).
template <class Src>
__device__ __forceinline__ uint32_t ragged_root_count(const Src& src, const OpProg& d, const uint8_t* aux, uint32_t s,
                                                      uint32_t e) {
  const bool multi = d.flags & F_MULTI;
  if (d.kind != OP_FILTER) return count_commas(src, s, e) + 1u;  // multi-valued hash / bucket
  const uint8_t* pre = aux + d.aux_off;
  const uint32_t plen = d.aux_len;
  uint32_t cnt = 0, k = 0;
  bool match = true;
  for_each_byte(src, s, e, [&](uint32_t b) {
    if (multi && b == ',') {
      cnt += (match && k >= plen) ? 1u : 0u;
      k = 0; match = true;
    } else {
      if (k < plen && b != pre[k]) match = false;
      ++k;
    }
  });
  cnt += (match && k >= plen) ? 1u : 0u;
  return cnt;
}

// Writes the signs of a ragged root operator (not n-gram) on [s, e) to dst[0 .. count).
template <class Src>
__device__ __forceinline__ void ragged_root_emit(const Src& src, const OpProg& d, const uint8_t* aux, uint32_t s,
                                                 uint32_t e, uint64_t* dst, uint32_t& malformed) {
  const bool multi = d.flags & F_MULTI;
  if (d.kind == OP_HASH) {  // a ragged hash is always multi-valued
    uint64_t h = d.key;
    const uint64_t key = d.key;
    for_each_byte(src, s, e, [&](uint32_t b) {
      if (b == ',') { *dst++ = h; h = key; }
      else h = (h ^ b) * kPrime;
    });
    *dst = h;
  } else if (d.kind == OP_FILTER) {
    const uint8_t* pre = aux + d.aux_off;
    const uint32_t plen = d.aux_len;
    const uint64_t key = d.key;
    uint64_t h = key;
    uint32_t k = 0;
    bool match = true;
    for_each_byte(src, s, e, [&](uint32_t b) {
      if (multi && b == ',') {
        if (match && k >= plen) *dst++ = h;
        h = key; k = 0; match = true;
      } else {
        if (k < plen && b != pre[k]) match = false;
        h = (h ^ b) * kPrime;
        ++k;
      }
    });
    if (match && k >= plen) *dst = h;
  } else {  // OP_BUCKET, multi-valued
    NumState ns;
    for_each_byte(src, s, e, [&](uint32_t b) {
      if (b == ',') {
        *dst++ = bucket_sign(d, aux, ns, malformed);
        ns = NumState();
      } else ns.step(b);
    });
    *dst = bucket_sign(d, aux, ns, malformed);
  }
}

// ------------------------------------------------------------ one pass of a tile
// Inclusive prefix sum inside groups of T neighbouring lanes.
__device__ __forceinline__ uint32_t group_incl_scan(uint32_t v, uint32_t T) {
  const uint32_t r = lane_id() & (T - 1u);
  for (uint32_t d = 1; d < T; d <<= 1) {
    const uint32_t t = __shfl_up(v, d, 64);
    if (r >= d) v += t;
  }
  return v;
}

// Runs every layer on the nb records of one pass.  g_first is the batch-wide
// index of the pass's first record.  WRITE = false stops after the counts.
template <bool WRITE, class Src>
__device__ void run_pass(const TileParams& P, const Sh& sh, const Src& src, uint32_t nb, uint64_t g_first,
                         uint32_t& malformed, bool& overflow) {
  const uint32_t T = 1u << P.log2T, G = 64u >> P.log2T;  // G operators per wavefront at a time
  const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const uint32_t r = lane & (T - 1u), og = lane >> P.log2T;
  const bool live = r < nb;
  const uint64_t g = g_first + r;
  const uint64_t R = P.n_records;
  constexpr uint32_t kWaves = kTileThreads / 64;

  // ---- counts of the ragged operators, then their positions inside the tile
  if (P.n_ragged) {
    for (uint32_t list = TL_RAGROOT; list <= TL_NGRAM; ++list) {
      const uint32_t lb = sh.list_begin[list], m = sh.list_begin[list + 1] - lb;
      for (uint32_t base = wave * G; base < m; base += kWaves * G) {
        const uint32_t i = base + og;
        if (i >= m) continue;
        const OpProg& d = sh.prog[sh.lists[lb + i]];
        uint32_t c = 0;
        if (live) {
          uint32_t s, e;
          src.span(r, d.field, s, e);
          if (d.kind == OP_NGRAM) c = e - s >= d.aux_len ? e - s - d.aux_len + 1u : 0u;
          else c = ragged_root_count(src, d, sh.aux, s, e);
        }
        if (c > kMaxCount) overflow = true;
        sh.cnt[d.rag_row * T + r] = c;
      }
    }
    __syncthreads();
    FBX_MARK(4);
    // later layers: counts follow from the inputs' counts, record by record, in spec order
    if (P.n_rnr) {
      if (tid < T) {
        for (uint32_t k = 0; k < P.n_rnr; ++k) {
          const OpProg& d = sh.prog[sh.rnr[k]];
          const OpProg& da = sh.prog[d.a];
          const OpProg& db = sh.prog[d.b];
          const uint64_t ca = da.arity ? da.arity : sh.cnt[da.rag_row * T + tid];
          const uint64_t cb = db.arity ? db.arity : sh.cnt[db.rag_row * T + tid];
          const uint64_t c = d.kind == OP_CROSS ? ca * cb : ca + cb;
          if (c > kMaxCount) overflow = true;
          sh.cnt[d.rag_row * T + tid] = tid < nb ? (uint32_t)c : 0u;
        }
      }
      __syncthreads();
    }
    for (uint32_t base = wave * G; base < P.n_ragged; base += kWaves * G) {
      const uint32_t row = base + og;
      const bool ok = row < P.n_ragged;
      const uint32_t v = ok ? sh.cnt[row * T + r] : 0u;
      const uint32_t incl = group_incl_scan(v, T);
      if (ok) {
        const uint32_t before = sh.run[row];
        sh.start[row * T + r] = before + incl - v;
        if (r == T - 1u) sh.run[row] = before + incl;
      }
    }
    __syncthreads();
    FBX_MARK(5);
  }
  if (!WRITE) return;

  // ---- layer 1
  // single-valued hashes and buckets: one sign per record
  for (uint32_t list = TL_HASH1; list <= TL_BUCKET1; ++list) {
    const uint32_t lb = sh.list_begin[list], m = sh.list_begin[list + 1] - lb;
    for (uint32_t base = wave * G; base < m; base += kWaves * G) {
      const uint32_t i = base + og;
      if (i >= m || !live) continue;
      const OpProg& d = sh.prog[sh.lists[lb + i]];
      uint32_t s, e;
      src.span(r, d.field, s, e);
      const uint64_t v = single_sign(src, d, sh.aux, s, e, malformed);
      reinterpret_cast<uint64_t*>(d.values)[g] = v;
      if (d.stage != kNoRow) sh.stage[d.stage * T + r] = v;
    }
  }
  FBX_MARK(6);
  // ragged root operators other than n-grams: a lane writes its record's list
  {
    const uint32_t lb = sh.list_begin[TL_RAGROOT], m = sh.list_begin[TL_RAGROOT + 1] - lb;
    for (uint32_t base = wave * G; base < m; base += kWaves * G) {
      const uint32_t i = base + og;
      if (i >= m || !live) continue;
      const OpProg& d = sh.prog[sh.lists[lb + i]];
      const uint64_t first = sh.base[d.rag_row] + sh.start[d.rag_row * T + r];
      if (d.flags & F_EMIT) {
        uint64_t* off = reinterpret_cast<uint64_t*>(d.offsets);
        off[g] = first;
        if (g + 1 == R) off[R] = first + sh.cnt[d.rag_row * T + r];
      }
      uint32_t s, e;
      src.span(r, d.field, s, e);
      ragged_root_emit(src, d, sh.aux, s, e, reinterpret_cast<uint64_t*>(d.values) + first, malformed);
    }
  }
  FBX_MARK(7);
  // n-grams: the lanes of a wavefront run over the grams of one record at a time
  {
    const uint32_t lb = sh.list_begin[TL_NGRAM], m = sh.list_begin[TL_NGRAM + 1] - lb;
    for (uint32_t i = 0; i < m; ++i) {
      const OpProg& d = sh.prog[sh.lists[lb + i]];
      const uint32_t n = d.aux_len;
      uint64_t* vals = reinterpret_cast<uint64_t*>(d.values);
      for (uint32_t rr = wave; rr < nb; rr += kWaves) {
        uint32_t s, e;
        src.span(rr, d.field, s, e);
        const uint32_t ng = sh.cnt[d.rag_row * T + rr];
        const uint64_t first = sh.base[d.rag_row] + sh.start[d.rag_row * T + rr];
        if (lane == 0 && (d.flags & F_EMIT)) {
          uint64_t* off = reinterpret_cast<uint64_t*>(d.offsets);
          off[g_first + rr] = first;
          if (g_first + rr + 1 == R) off[R] = first + ng;
        }
        const uint64_t key = d.key;
        for (uint32_t q = lane; q < ng; q += 64) vals[first + q] = hash_span(src, s + q, s + q + n, key);
      }
    }
  }

  FBX_MARK(8);
  // ---- later layers
  for (uint32_t layer = 2; layer <= P.n_layers; ++layer) {
    __syncthreads();  // the layer barrier: every sign of the layer before is in place
    FBX_MARK(9);
    // crosses of two single signs, both on chip
    {
      const uint32_t list = TL_LAYER + 2u * (layer - 2u);
      const uint32_t lb = sh.list_begin[list], m = sh.list_begin[list + 1] - lb;
      for (uint32_t base = wave * G; base < m; base += kWaves * G) {
        const uint32_t i = base + og;
        if (i >= m || !live) continue;
        const OpProg& d = sh.prog[sh.lists[lb + i]];
        const uint64_t a = sh.stage[d.aux_off * T + r], b = sh.stage[d.aux_len * T + r];
        const uint64_t v = mix64(mix64(a + d.key) + b);
        reinterpret_cast<uint64_t*>(d.values)[g] = v;
        if (d.stage != kNoRow) sh.stage[d.stage * T + r] = v;
      }
    }
    FBX_MARK(10);
    // every other cross or concat: inputs are lists in the arrays this workgroup wrote
    {
      const uint32_t list = TL_LAYER + 2u * (layer - 2u) + 1u;
      const uint32_t lb = sh.list_begin[list], m = sh.list_begin[list + 1] - lb;
      for (uint32_t base = wave * G; base < m; base += kWaves * G) {
        const uint32_t i = base + og;
        if (i >= m || !live) continue;
        const OpProg& d = sh.prog[sh.lists[lb + i]];
        const OpProg& da = sh.prog[d.a];
        const OpProg& db = sh.prog[d.b];
        const uint64_t* pa;
        const uint64_t* pb;
        uint32_t na, nbv;
        if (da.arity) { na = da.arity; pa = reinterpret_cast<const uint64_t*>(da.values) + g * da.arity; }
        else {
          na = sh.cnt[da.rag_row * T + r];
          pa = reinterpret_cast<const uint64_t*>(da.values) + sh.base[da.rag_row] + sh.start[da.rag_row * T + r];
        }
        if (db.arity) { nbv = db.arity; pb = reinterpret_cast<const uint64_t*>(db.values) + g * db.arity; }
        else {
          nbv = sh.cnt[db.rag_row * T + r];
          pb = reinterpret_cast<const uint64_t*>(db.values) + sh.base[db.rag_row] + sh.start[db.rag_row * T + r];
        }
        uint64_t* dst;
        if (d.arity) {
          dst = reinterpret_cast<uint64_t*>(d.values) + g * d.arity;
        } else {
          const uint64_t first = sh.base[d.rag_row] + sh.start[d.rag_row * T + r];
          dst = reinterpret_cast<uint64_t*>(d.values) + first;
          if (d.flags & F_EMIT) {
            uint64_t* off = reinterpret_cast<uint64_t*>(d.offsets);
            off[g] = first;
            if (g + 1 == R) off[R] = first + sh.cnt[d.rag_row * T + r];
          }
        }
        if (d.kind == OP_CROSS) {
          for (uint32_t x = 0; x < na; ++x) {
            const uint64_t ma = mix64(pa[x] + d.key);
            for (uint32_t y = 0; y < nbv; ++y) *dst++ = mix64(ma + pb[y]);
          }
        } else {
          for (uint32_t x = 0; x < na; ++x) *dst++ = pa[x];
          for (uint32_t y = 0; y < nbv; ++y) *dst++ = pb[y];
        }
      }
    }
    FBX_MARK(11);
  }
}

// ------------------------------------------------------------------- kernel
// Copies n bytes (a multiple of 4) from memory into LDS, all lanes taking part.
__device__ __forceinline__ void copy_table(uint8_t* dst, const void* src, uint32_t n) {
  const uint32_t* s32 = reinterpret_cast<const uint32_t*>(src);
  uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
  for (uint32_t i = threadIdx.x; i < (n >> 2); i += kTileThreads) d32[i] = s32[i];
}

// Workgroups are persistent: each copies the plan tables into LDS once and then
// takes tiles off a shared counter, in increasing order, until none is left.
template <bool WRITE>
__global__ __launch_bounds__(kTileThreads) void k_tile(TileParams P) {
  __shared__ uint32_t s_err;
  __shared__ uint32_t s_len;
  __shared__ uint32_t s_tile;
  const Sh sh = views(P);
  const uint32_t tid = threadIdx.x;
  const uint32_t T = 1u << P.log2T;
  if (tid == 0) s_err = P.ctrl->err;  // set by an earlier kernel of this call: nothing may be written
  copy_table(smem + P.o_prog, P.prog, P.n_ops * (uint32_t)sizeof(OpProg));
  copy_table(smem + P.o_lists, P.lists, P.n_ops * 4u);
  copy_table(smem + P.o_lbeg, P.list_begin, (P.n_lists + 1u) * 4u);
  copy_table(smem + P.o_rnr, P.rnr, P.n_rnr * 4u);
  copy_table(smem + P.o_aux, P.aux, P.aux_bytes);
#ifdef FBX_TILE_PROF
  if (tid < 16) s_prof[tid] = 0;
  if (tid == 0) s_prof_last = clock64();
#endif
  __syncthreads();
  if (s_err) return;
  FBX_MARK(0);

  uint32_t malformed = 0;
  bool overflow = false;
  for (;;) {
    if (tid == 0) s_tile = atomicAdd(&P.ctrl->ticket[WRITE ? 1 : 0], 1u);
    __syncthreads();
    const uint32_t tile = s_tile;
    if (tile >= P.n_tiles) break;
    const uint64_t g0 = (uint64_t)tile << P.log2T;
    const uint32_t nrec = (uint32_t)min((uint64_t)T, P.n_records - g0);
    if (tid <= nrec) sh.off[tid] = P.rec_off[g0 + tid];
    for (uint32_t row = tid; row < P.n_ragged; row += kTileThreads) {
      sh.run[row] = 0;
      if (WRITE) sh.base[row] = P.tile_base[(uint64_t)row * P.n_tiles + tile];
    }
    __syncthreads();
    uint32_t bad = 0;
    if (tid < nrec) {
      const uint64_t a = sh.off[tid], b = sh.off[tid + 1];
      if (a > b || b > P.raw_len) bad = CE_OFFSETS;
      else if (b - a >= (1ull << 31)) bad = CE_TILE;
    }
    if (__syncthreads_or((int)bad)) {
      if (bad) atomicOr(&P.ctrl->err, bad);
      break;  // the call fails: no point in working off the other tiles
    }
    FBX_MARK(1);

    uint32_t r0 = 0;
    while (r0 < nrec) {  // one turn per pass; all conditions are uniform over the workgroup
      const uint64_t o0 = sh.off[r0];
      const uintptr_t addr0 = reinterpret_cast<uintptr_t>(P.raw) + o0;
      const uint32_t delta = (uint32_t)(addr0 & 15u);
      // the pass takes records r0 .. r1-1: as many as fit the LDS section
      uint32_t lo = r0, hi = nrec;
      while (lo < hi) {
        const uint32_t mid = (lo + hi + 1u) >> 1;
        if (sh.off[mid] - o0 + delta <= (uint64_t)P.raw_cap) lo = mid; else hi = mid - 1u;
      }
      const uint32_t r1 = lo;
      if (r1 > r0) {
        const uint32_t nb = r1 - r0;
        const uint32_t nbytes = delta + (uint32_t)(sh.off[r1] - o0);
        const uint32_t nchunks = (nbytes + 15u) >> 4;
        const uintptr_t a0 = addr0 - delta;
        const uintptr_t ok_lo = reinterpret_cast<uintptr_t>(P.raw), ok_hi = ok_lo + P.raw_len;
        for (uint32_t c = tid; c < nchunks; c += kTileThreads) {
          const uintptr_t ca = a0 + 16u * c;
          u32x4 v;
          if (ca >= ok_lo && ca + 16u <= ok_hi) {
            v = *reinterpret_cast<const u32x4*>(ca);
          } else {  // the chunk straddles an end of the caller's buffer: take what exists byte by byte
            uint32_t w[4] = {0, 0, 0, 0};
            for (uint32_t i = 0; i < 16; ++i) {
              const uintptr_t bi = ca + i;
              if (bi >= ok_lo && bi < ok_hi)
                w[i >> 2] |= (uint32_t)*reinterpret_cast<const uint8_t*>(bi) << (8u * (i & 3u));
            }
            v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
          }
          *reinterpret_cast<u32x4*>(sh.raw + kRawPad + 16u * c) = v;
        }
        if (tid < nb) {
          sh.rs[tid] = kRawPad + delta + (uint32_t)(sh.off[r0 + tid] - o0);
          sh.re[tid] = kRawPad + delta + (uint32_t)(sh.off[r0 + tid + 1] - o0);
        }
        __syncthreads();
        // one trailing newline is not part of the record
        if (tid < nb) {
          const uint32_t e = sh.re[tid];
          if (e > sh.rs[tid] && sh.raw[e - 1u] == '\n') sh.re[tid] = e - 1u;
        }
        __syncthreads();
        FBX_MARK(2);
        tokenize(P, sh, nb);
        __syncthreads();
        FBX_MARK(3);
        LdsSrc src{sh.raw, sh.rows, P.row_stride};
        run_pass<WRITE>(P, sh, src, nb, g0 + r0, malformed, overflow);
        r0 = r1;
      } else {
        // record r0 alone exceeds the section: it is read in place
        const uint64_t len64 = sh.off[r0 + 1] - o0;
        if (tid == 0) {
          uint32_t len = (uint32_t)len64;
          if (len && P.raw[o0 + len - 1u] == '\n') --len;
          s_len = len;
        }
        __syncthreads();
        GlobalSrc src{P.raw + o0, s_len};
        run_pass<WRITE>(P, sh, src, 1u, g0 + r0, malformed, overflow);
        r0 += 1u;
      }
      __syncthreads();  // the sections are reused by the next pass
      FBX_MARK(12);
    }
    if (!WRITE) {
      for (uint32_t row = tid; row < P.n_ragged; row += kTileThreads)
        P.tile_cnt[(uint64_t)row * P.n_tiles + tile] = sh.run[row];
    }
    __syncthreads();  // s_tile and the tile's sections are rewritten next
  }

#ifdef FBX_TILE_PROF
  __syncthreads();
  if (tid < 16 && P.prof) atomicAdd(reinterpret_cast<unsigned long long*>(P.prof) + tid + (WRITE ? 16 : 0), s_prof[tid]);
#endif
  if (!WRITE) {
    if (overflow) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
  } else {
    for (int d = 32; d >= 1; d >>= 1) malformed += __shfl_xor(malformed, d, 64);
    if (lane_id() == 0 && malformed)
      atomicAdd(reinterpret_cast<unsigned long long*>(&P.ctrl->n_malformed), (unsigned long long)malformed);
  }
}

}  // namespace

// ----------------------------------------------------------- launch wrappers
uint32_t tile_max_lds() {
  static uint32_t cached = 0;
  if (!cached) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
      cached = (uint32_t)v;
    else
      cached = 64u * 1024u;
  }
  return cached;
}

hipError_t launch_tile(const TileParams& P, int write, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  const void* fn = write ? reinterpret_cast<const void*>(&k_tile<true>) : reinterpret_cast<const void*>(&k_tile<false>);
  if (P.lds_bytes > 48u * 1024u) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)P.lds_bytes);
    if (e != hipSuccess) return e;
  }
  const uint32_t grid = std::min(P.n_tiles, P.grid);
  if (write) hipLaunchKernelGGL(k_tile<true>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, P);
  else hipLaunchKernelGGL(k_tile<false>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, P);
  return hipGetLastError();
}

uint32_t tile_cu_count() {
  static uint32_t cached = 0;
  if (!cached) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cached = (uint32_t)v;
    else
      cached = 256u;
  }
  return cached;
}

}  // namespace fbx
