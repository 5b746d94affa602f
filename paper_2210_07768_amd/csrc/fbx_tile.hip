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
//     share a record, find its tabs sixteen bytes at a time and write a table of
//     field ends (16-bit LDS positions).  No per-thread array is allocated; the
//     table has one entry per (record, field).  The same routine splits the item
//     lists of multi-valued fields at their commas.
//  3. Layer 1: lanes are (record, operator) pairs.  A lane looks up its field in
//     the table and hashes / parses it out of LDS; T neighbouring lanes hold T
//     consecutive records of one operator, so a slot is written in runs of 8 T
//     bytes.  Signs that a later operator needs stay in an LDS table as well.
//  4. Later layers run after the barrier: crosses of two single signs out of that
//     table; list operators with one lane per output sign, reading lists from
//     the arrays this workgroup wrote.  A cross of a multi-valued hash with a
//     single sign is computed by the lane that hashes the item.
//  5. Ragged slots: the per-record counts of the tile are found first, then
//     turned into positions by a prefix sum over the tile's records on top of
//     the tile's base.  The base comes from a counting launch of this same
//     kernel and a scan over tiles, or, in the one-launch mode, from the words
//     that the tiles before this one have published (see lb_place_row), or,
//     where the caller does not need record order, from one atomic add on the
//     operator's running total (place_by_arrival).
//  6. Workgroups are persistent and software-pipelined: while a tile is worked
//     on, the ticket and the record offsets of the next tile are fetched and one
//     byte of every line of its text is touched, so that the text is on its way
//     into the cache when the tile's turn comes.
//
// A tile whose text does not fit the LDS section is worked off in several
// passes of fewer records; a single record that does not fit alone is walked
// straight from memory, one lane per operator (slow, rare, same results).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "fbx_arena.h"
#include "fbx_device.h"
#include "fbx_split.h"

// How a tile of 64 records runs its single-sign operators (kernels compiled for a plan only): 0 as any
// other tile, 1 one operator per wavefront with its numbers from the program table, 2 the same as
// straight-line code generated for the plan (FBX_GEN_L1, FBX_GEN_X11).
#ifndef FBX_LANE_OPS
#define FBX_LANE_OPS 0
#endif
#ifndef FBX_EXP
#define FBX_EXP 0
#endif


namespace fbx {
namespace {

constexpr uint32_t kNoRow = 0xffffffffu;
constexpr uint64_t kPrime = 0x100000001b3ull;
constexpr uint32_t kMaxCount = 0x3ffffffu;  // signs per record and operator


// Pointers the compiler knows to be global memory (plain global loads and stores
// instead of flat ones, which would also wait on the LDS counter).
#define FBX_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ FBX_GLOBAL T* gptr(uint64_t addr) { return reinterpret_cast<FBX_GLOBAL T*>(addr); }
template <class T>
__device__ __forceinline__ FBX_GLOBAL T* gptr(T* p) { return reinterpret_cast<FBX_GLOBAL T*>(reinterpret_cast<uintptr_t>(p)); }
using G64 = FBX_GLOBAL uint64_t*;
using CG64 = const FBX_GLOBAL uint64_t*;
// Memory that no kernel of the call writes while this one runs (the per-call operator programs): loads
// through such a pointer at an address all lanes share go through the scalar unit.
#define FBX_CONSTANT __attribute__((address_space(4)))
template <class T>
__device__ __forceinline__ const FBX_CONSTANT T* cptr(const T* p) {
  return reinterpret_cast<const FBX_CONSTANT T*>(reinterpret_cast<uintptr_t>(p));
}

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
#define FBX_SKIP(bit) (P.dbg & (bit))
#define FBX_TALLY(n, v)                                         \
  do {                                                          \
    if (lane_id() == 0) atomicAdd(&s_prof[n], (unsigned long long)(v)); \
  } while (0)
#else
#define FBX_TALLY(n, v) do {} while (0)
#define FBX_MARK(n) do {} while (0)
#define FBX_SKIP(bit) false
#endif

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}


// Views of the LDS sections of one workgroup.
#ifdef FBX_FIXED_MODE
// The bounds of the plan's work lists and the first entry of every layer in the table of derived
// counts: small tables of the plan, literals in a kernel compiled for it.
__device__ __forceinline__ uint32_t fixed_list_begin(uint32_t i) {
  constexpr uint32_t t[] = FBX_FIXED_LIST_BEGIN;
  return t[i];
}
__device__ __forceinline__ uint32_t fixed_rnr_head(uint32_t i) {
  constexpr uint32_t t[] = FBX_FIXED_RNR_HEAD;
  return t[i];
}
#endif

struct Sh {
  uint64_t* off;    // [2][T + 1] record offsets of this tile and of the next one
  uint32_t* rs;     // [T] LDS position of the first byte of a staged record
  uint32_t* re;     // [T] LDS position one past its last byte (newline dropped)
  uint16_t* rows;   // [T][row_stride]: row[0] = rs - 1, row[1 + k] = end of field k
  uint8_t* raw;     // staged text; byte 0 of the staged range sits at kRawPad + (address & 15)
  uint64_t* stage;  // [n_stage][T] single signs kept for later layers
  uint32_t* cnt;    // [n_ragged][T] signs of a ragged operator per record
  uint32_t* start;  // [n_ragged][T] their first position, relative to the tile's base
  uint32_t* run;    // [n_ragged] signs of the tile's earlier passes
  uint64_t* base;   // [n_ragged] the tile's base in the operator's values array
  uint32_t* tot;    // [n_ragged] signs of this pass
  uint64_t* cap;    // [n_ragged] signs the operator's array has room for (one-launch mode)
  uint32_t* gfirst; // [n_ops] list operators of layers >= 2, by program position: first sign among the signs of the layer's list operators in this pass
  uint32_t* gtot;   // [n_layers + 1] signs of all list operators of a layer in this pass
  uint32_t* ioff;   // [n_mh + 1] first item of every multi-valued hash among the pass's items
  uint16_t* ctab;   // [n_mh][T][item_cap] comma positions of the multi-valued hash fields
  // plan tables, copied once per workgroup so that no lane waits on memory for a descriptor
  const OpProg* prog;          // [n_ops], in the order of the work lists
  const uint32_t* list_begin;
  const uint32_t* rnr;         // how the counts of the ragged operators of layers >= 2 follow from their inputs'
  const uint8_t* aux;          // bucket boundaries and filter prefixes
  // bounds of work list i; first entry of layer i + 2 in rnr (i < n_layers)
#ifdef FBX_FIXED_MODE
  __device__ __forceinline__ uint32_t lbeg(uint32_t i) const { return fixed_list_begin(i); }
  __device__ __forceinline__ uint32_t rnr_head(uint32_t i) const { return fixed_rnr_head(i); }
#else
  // (the bounds of the lists that every plan has are fetched once per kernel and stay in scalar
  // registers: a unit of work then starts without a look-up it would have to wait for)
  uint32_t lb[TL_LAYER + 1];
  __device__ __forceinline__ uint32_t lbeg(uint32_t i) const {
    return (__builtin_constant_p(i) && i <= (uint32_t)TL_LAYER) ? lb[i] : list_begin[i];
  }
  __device__ __forceinline__ uint32_t rnr_head(uint32_t i) const { return rnr[i]; }
#endif
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
  s.tot = reinterpret_cast<uint32_t*>(smem + P.o_tot);
  s.cap = reinterpret_cast<uint64_t*>(smem + P.o_cap);
  s.gfirst = reinterpret_cast<uint32_t*>(smem + P.o_gfirst);
  s.gtot = reinterpret_cast<uint32_t*>(smem + P.o_gtot);
  s.ioff = reinterpret_cast<uint32_t*>(smem + P.o_ioff);
  s.ctab = reinterpret_cast<uint16_t*>(smem + P.o_ctab);
  s.prog = reinterpret_cast<const OpProg*>(smem + P.o_prog);
  s.list_begin = reinterpret_cast<const uint32_t*>(smem + P.o_lbeg);
  s.rnr = reinterpret_cast<const uint32_t*>(smem + P.o_rnr);
  s.aux = smem + P.o_aux;
  return s;
}

// ------------------------------------------------------------ byte sources
// Where a lane reads record bytes from.  Positions are 32-bit.
// One-launch mode: true for a ragged row whose signs before a tile follow from another row's
// (the plan's table of such rows: PlanHost::alias_at); such a row publishes nothing and is placed
// along with the row it follows.
__device__ __forceinline__ bool row_follows(const TileParams& P, const Sh& sh, uint32_t row) {
  return P.n_alias != 0u && sh.rnr[P.alias_at + 3u * row] != kNoAlias;
}

struct LdsSrc {
  static constexpr bool kTable = true;  // positions fit the 16-bit comma table
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
  static constexpr bool kTable = false;
  const FBX_GLOBAL uint8_t* rec;
  uint32_t len;  // newline dropped
  __device__ __forceinline__ uint32_t byte(uint32_t p) const { return rec[p]; }
  __device__ __forceinline__ void span(uint32_t, uint32_t k, uint32_t& s, uint32_t& e) const {
    uint32_t p = 0, f = 0;
    // eight bytes at a time while the field lies further on (a load at any address: the compiler
    // emits what the target allows for it), then byte by byte
    while (f < k && p + 8u <= len) {
      uint64_t w;
      __builtin_memcpy(&w, rec + p, 8);
      const uint32_t n = __popc(eq_flags((uint32_t)w, kTabs)) + __popc(eq_flags((uint32_t)(w >> 32), kTabs));
      if (f + n >= k) break;  // the tab in front of the field is among these eight
      f += n;
      p += 8u;
    }
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
// (eq_flags, group_prefix and split_bytes: fbx_split.h)

// Field table of the staged records.  kTileThreads / T lanes (at most 64) share a
// record and place its tabs.  Entries from the record's tab count on hold the
// record's end.
__device__ __forceinline__ void tokenize(const TileParams& P, const Sh& sh, uint32_t nb) {
  const uint32_t tid = thread_id();
  constexpr uint32_t kLogThreads = kTileThreads == 1024 ? 10u : (kTileThreads == 512 ? 9u : 8u);
  const uint32_t lg = kLogThreads - P.log2T < 6u ? kLogThreads - P.log2T : 6u;  // log2 of the lanes per record
  const uint32_t gsz = 1u << lg;
  const uint32_t j = tid & (gsz - 1u);
  const uint32_t r = tid >> lg;
  const uint32_t F = P.n_fields;
  const bool act = r < nb;
  uint32_t rs = 0, re = 0;
  if (act) {
    rs = sh.rs[r]; re = sh.re[r];
    if (re > rs && sh.raw[re - 1u] == '\n') --re;  // one trailing newline is not part of the record
  }
  uint16_t* row = sh.rows + r * P.row_stride;
  const uint32_t total = split_bytes(sh.raw, rs, re, act, kTabs, lg, j, F, [&](uint32_t k, uint32_t pos) {
    row[1u + k] = (uint16_t)pos;
  });
  if (!act) return;
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
// Calls f(word, K) for the bytes [s, e) in order: the byte is byte K (a compile-time constant,
// passed as std::integral_constant) of the 32-bit word.
template <class F>
__device__ __forceinline__ void for_each_byte_of_word(const LdsSrc& src, uint32_t s, uint32_t e, F&& f) {
  uint32_t p = s;
  while (p < e) {
    uint32_t x0, x1;
    window8(src, p, x0, x1);
    const uint32_t n = e - p < 8u ? e - p : 8u;
#define FBX_STEP(J, X) if (n > (uint32_t)J) { f(X, std::integral_constant<int, (J & 3)>());
    FBX_STEP(0, x0) FBX_STEP(1, x0) FBX_STEP(2, x0) FBX_STEP(3, x0)
    FBX_STEP(4, x1) FBX_STEP(5, x1) FBX_STEP(6, x1) FBX_STEP(7, x1)
    }}}}}}}}
#undef FBX_STEP
    p += n;
  }
}
template <class F>
__device__ __forceinline__ void for_each_byte(const LdsSrc& src, uint32_t s, uint32_t e, F&& f) {
  for_each_byte_of_word(src, s, e, [&](uint32_t w, auto k) { f((w >> (8 * decltype(k)::value)) & 0xffu); });
}

template <class F>
__device__ __forceinline__ void for_each_byte(const GlobalSrc& src, uint32_t s, uint32_t e, F&& f) {
  for (uint32_t p = s; p < e; ++p) f(src.byte(p));
}
template <class F>
__device__ __forceinline__ void for_each_byte_of_word(const GlobalSrc& src, uint32_t s, uint32_t e, F&& f) {
  for (uint32_t p = s; p < e; ++p) f(src.byte(p), std::integral_constant<int, 0>());
}

// a ^ (byte K of w), in one instruction (sub-dword operand selection)
template <int K>
__device__ __forceinline__ uint32_t xor_byte(uint32_t a, uint32_t w) {
  uint32_t r;
  if (K == 0) asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(a), "v"(w));
  else if (K == 1) asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(a), "v"(w));
  else if (K == 2) asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(a), "v"(w));
  else asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(a), "v"(w));
  return r;
}

// FNV-1a over the bytes [s, e) from state h: h = (h ^ b) * (2^40 + 435) per byte.  Only the low
// word's product needs the wide multiply-add; the high word's own terms, 435 hi + (lo << 8), go
// in as its addend.
template <class Src>
__device__ __forceinline__ uint64_t hash_span(const Src& src, uint32_t s, uint32_t e, uint64_t h) {
  static_assert(kPrime == ((1ull << 40) | 435ull), "FNV-1a prime");
  uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
  for_each_byte_of_word(src, s, e, [&](uint32_t w, auto k) {
    lo = xor_byte<decltype(k)::value>(lo, w);
    const uint32_t top = hi * 435u + (lo << 8);
    uint64_t r, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(r), "=s"(carry) : "v"(lo), "s"(435u), "v"((uint64_t)top << 32));
    lo = (uint32_t)r;
    hi = (uint32_t)(r >> 32);
  });
  return ((uint64_t)hi << 32) | lo;
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

// Position of the first comma in [p, e), or e.
__device__ __forceinline__ uint32_t next_comma(const LdsSrc& src, uint32_t p, uint32_t e) {
  while (p < e) {
    uint32_t x0, x1;
    window8(src, p, x0, x1);
    const uint32_t f0 = zero_exact(x0 ^ 0x2c2c2c2cu), f1 = zero_exact(x1 ^ 0x2c2c2c2cu);
    const uint32_t i0 = ((uint32_t)__ffs((int)f0) - 1u) >> 3, i1 = 4u + (((uint32_t)__ffs((int)f1) - 1u) >> 3);
    const uint32_t idx = f0 ? i0 : (f1 ? i1 : 8u);
    p += idx;
    if (idx < 8u) break;
  }
  return p < e ? p : e;
}

__device__ __forceinline__ uint32_t next_comma(const GlobalSrc& src, uint32_t p, uint32_t e) {
  while (p < e && src.byte(p) != ',') ++p;
  return p;
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

// The same grammar over a staged token [s, e) without a loop over its bytes.  The token's first
// sixteen bytes are fetched at once; a bit mask of the bytes that are not digits gives the ends of
// the integer part and of the fraction (count trailing zeros); up to eight integer digits and the
// first six fraction digits are converted four at a time (digit pairs by one multiply-add, pairs
// of pairs by another).  Tokens longer than sixteen bytes or integer parts longer than eight
// digits (rare) take the byte-by-byte state machine.  Value and malformed flag as NumState's.
__device__ __forceinline__ uint32_t four_digits(uint32_t w) {  // bytes 0..3 hold digit values, byte 0 the most significant
  const uint32_t t = w * 10u + (w >> 8);                       // byte 0: d0 * 10 + d1, byte 2: d2 * 10 + d3 (no carries: <= 99)
  return (t & 0xffu) * 100u + ((t >> 16) & 0xffu);
}
__device__ __forceinline__ int64_t parse_micro(const LdsSrc& src, uint32_t s, uint32_t e, bool& bad) {
  const uint32_t n = e - s;
  uint32_t x0, x1, x2, x3;
  window8(src, s, x0, x1);
  window8(src, s + 8u, x2, x3);
  // bit i: byte i is not a digit (bytes at and beyond n count as such)
  auto not_digit = [](uint32_t w) -> uint32_t {
    const uint32_t t = w ^ 0x30303030u;  // '0'..'9' become 0..9
    return (((t & 0x7f7f7f7fu) + 0x76767676u) | t) & 0x80808080u;
  };
  uint32_t lo8 = __builtin_amdgcn_udot4(not_digit(x0), 0x08040201u, 0u, false);
  lo8 = __builtin_amdgcn_udot4(not_digit(x1), 0x80402010u, lo8, false);
  uint32_t hi8 = __builtin_amdgcn_udot4(not_digit(x2), 0x08040201u, 0u, false);
  hi8 = __builtin_amdgcn_udot4(not_digit(x3), 0x80402010u, hi8, false);
  const uint32_t nd = (((lo8 | (hi8 << 8)) >> 7) | (n >= 16u ? 0x10000u : (~0u << n))) & 0x1ffffu;
  const uint32_t neg = (x0 & 0xffu) == '-' && n ? 1u : 0u;
  const uint32_t i1 = neg + (uint32_t)__builtin_ctz(nd >> neg);           // end of the integer part (<= 16)
  // the byte at i1, if it lies inside the token
  const uint32_t pick = i1 & 8u ? ((i1 & 4u) ? x3 : x2) : ((i1 & 4u) ? x1 : x0);
  const bool dot = i1 < n && i1 < 16u && ((pick >> (8u * (i1 & 3u))) & 0xffu) == '.';
  const uint32_t f0 = i1 + 1u;                                            // first byte of the fraction, if there is one
  const uint32_t i2 = dot ? f0 + (uint32_t)__builtin_ctz((nd >> f0) | (1u << (16u - min(f0, 16u)))) : i1;  // end of what fits the grammar
  const uint32_t ni = i1 - neg, nfd = dot ? i2 - f0 : 0u;
  if (n > 16u || ni > 8u || i2 > 16u) {  // beyond the window: byte by byte
    NumState ns;
    for_each_byte(src, s, e, [&](uint32_t b) { ns.step(b); });
    return ns.finish(bad);
  }
  bad = i2 < n || ni + nfd == 0u;
  // integer part: its ni bytes moved to the top of a 64-bit word, zeros (leading digits of value 0) below
  const uint64_t all_lo = ((uint64_t)x1 << 32) | x0, all_hi = ((uint64_t)x3 << 32) | x2;
  const uint64_t from_start = neg ? (all_lo >> 8) | (all_hi << 56) : all_lo;
  const uint64_t top = ni ? (from_start << (64u - 8u * ni)) & 0x0f0f0f0f0f0f0f0full : 0ull;
  const uint32_t ip = four_digits((uint32_t)top) * 10000u + four_digits((uint32_t)(top >> 32));
  // fraction: its first (up to six) bytes at the bottom of a word, zeros (trailing digits of value 0) above
  const uint32_t nf = min(nfd, 6u);
  uint64_t fr = f0 >= 8u ? all_hi >> (8u * min(f0 - 8u, 7u)) : (all_lo >> (8u * f0)) | (all_hi << (64u - 8u * f0));  // (f0 >= 1; at f0 = 16 nf is 0)
  fr &= 0x0f0f0f0f0f0f0f0full & ((1ull << (8u * nf)) - 1ull);
  const uint32_t h = (uint32_t)(fr >> 32);
  const uint32_t fp = four_digits((uint32_t)fr) * 100u + (((h * 10u + (h >> 8)) & 0xffu));
  uint64_t v = (uint64_t)ip * 1000000ull + fp;
  if (neg) v = 0ull - v;
  return (int64_t)v;
}
__device__ __forceinline__ int64_t parse_micro(const GlobalSrc& src, uint32_t s, uint32_t e, bool& bad) {
  NumState ns;
  for (uint32_t p = s; p < e; ++p) ns.step(src.byte(p));
  return ns.finish(bad);
}
// index = number of boundaries <= v; sign = mix64(key + index)
__device__ __forceinline__ uint64_t bucket_of(int64_t v, uint64_t key, const uint8_t* aux, uint32_t aux_off, uint32_t n_bounds) {
  const int64_t* b = reinterpret_cast<const int64_t*>(aux + aux_off);
  uint32_t lo = 0, hi = n_bounds;
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (b[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return mix64(key + lo);
}

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

// The prefix of a filter.  Its first eight bytes are fetched once and kept in two registers, with
// the masks of the bytes that count, so that a token is tested by comparing words; longer
// prefixes (rare) go on byte by byte in the table.
struct Prefix {
  const uint8_t* pre;
  uint32_t plen, lo, hi, mlo, mhi;
  __device__ __forceinline__ Prefix(const uint8_t* aux, const OpProg& d) : pre(aux + d.aux_off), plen(d.aux_len), lo(0), hi(0) {
#pragma unroll
    for (uint32_t k = 0; k < 8u; ++k) {
      const uint32_t b = k < plen ? pre[k] : 0u;
      if (k < 4u) lo |= b << (8u * k);
      else hi |= b << (8u * (k - 4u));
    }
    mlo = plen >= 4u ? ~0u : (1u << (8u * plen)) - 1u;
    mhi = plen <= 4u ? 0u : (plen >= 8u ? ~0u : (1u << (8u * (plen - 4u))) - 1u);
  }
};

// Whether the token [t, te) begins with the prefix.
__device__ __forceinline__ bool starts_with(const LdsSrc& src, uint32_t t, uint32_t te, const Prefix& pre) {
  if (te - t < pre.plen) return false;
  if (pre.plen == 0u) return true;
  uint32_t x0, x1;
  window8(src, t, x0, x1);
  bool ok = (((x0 ^ pre.lo) & pre.mlo) | ((x1 ^ pre.hi) & pre.mhi)) == 0u;
  for (uint32_t k = 8u; k < pre.plen && ok; ++k) ok = src.byte(t + k) == pre.pre[k];
  return ok;
}
__device__ __forceinline__ bool starts_with(const GlobalSrc& src, uint32_t t, uint32_t te, const Prefix& pre) {
  if (te - t < pre.plen) return false;
  bool ok = true;
  for (uint32_t k = 0; k < pre.plen && ok; ++k) ok = src.byte(t + k) == pre.pre[k];
  return ok;
}

// Calls f(t, te) for every token [t, te) of the field [s, e), in order: the field itself, or with
// multi its comma-separated parts (one more than it has commas, empty ones included).
template <class Src, class F>
__device__ __forceinline__ void for_each_token(const Src& src, uint32_t s, uint32_t e, bool multi, F&& f) {
  uint32_t t = s;
  for (;;) {
    const uint32_t te = multi ? next_comma(src, t, e) : e;
    f(t, te);
    if (te >= e) break;
    t = te + 1u;
  }
}

// Number of signs a ragged root operator (not n-gram) produces on [s, e).
template <class Src>
__device__ __forceinline__ uint32_t ragged_root_count(const Src& src, const OpProg& d, const uint8_t* aux, uint32_t s,
                                                      uint32_t e) {
  if (d.kind != OP_FILTER) return count_commas(src, s, e) + 1u;  // multi-valued hash / bucket
  const Prefix pre(aux, d);
  uint32_t cnt = 0;
  for_each_token(src, s, e, d.flags & F_MULTI, [&](uint32_t t, uint32_t te) { cnt += starts_with(src, t, te, pre) ? 1u : 0u; });
  return cnt;
}

// Writes the signs of a ragged root operator (not n-gram) on [s, e) to dst[0 .. count).
template <class Src>
__device__ __forceinline__ void ragged_root_emit(const Src& src, const OpProg& d, const uint8_t* aux, uint32_t s,
                                                 uint32_t e, G64 dst, uint32_t& malformed) {
  const bool multi = d.flags & F_MULTI;
  if (d.kind == OP_HASH) {  // a ragged hash is always multi-valued
    uint64_t h = d.key;
    const uint64_t key = d.key;
    for_each_byte(src, s, e, [&](uint32_t b) {
      if (b == ',') { *dst++ = h; h = key; }
      else h = (h ^ b) * kPrime;
    });
    *dst = h;
  } else if (d.kind == OP_FILTER) {  // only the tokens that pass are hashed
    const Prefix pre(aux, d);
    const uint64_t key = d.key;
    for_each_token(src, s, e, multi, [&](uint32_t t, uint32_t te) {
      if (starts_with(src, t, te, pre)) *dst++ = hash_span(src, t, te, key);
    });
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
  return group_prefix(v, 31u - (uint32_t)__clz((int)T), lane_id() & (T - 1u));
}

constexpr uint32_t kWaves = kTileThreads / 64;

// Work counters of a pass (cleared between passes): s_ctr[0] hands out the
// single-valued hash / bucket units of layer 1, which fill every phase that has
// idle wavefronts; s_ctr[1] the counting units, s_ctr[3] the ragged root units,
// s_ctr[4 + (l & 1)] the single crosses of layer l, s_ctr[7 + (l & 1)] its list operators.
// s_done: finished counting units.
__shared__ uint32_t s_ctr[9];
__shared__ uint32_t s_done;
__shared__ uint32_t s_good;   // MODE 2: the tile's bases are known and inside the arrays
__shared__ uint32_t s_absurd; // MODE 2: some lane saw a count beyond kMaxCount in this tile

// Next unit of a phase, the same for every lane of the wavefront.
__device__ __forceinline__ uint32_t grab_unit(uint32_t* ctr) {
  uint32_t u = 0;
  if (lane_id() == 0) u = atomicAdd(ctr, 1u);
  return __builtin_amdgcn_readfirstlane(u);
}
// Runs unit(u) for the units a wavefront gets of a phase with `total` units.  The next
// unit is asked for before the current one runs, so that the answer is there when needed.
template <class F>
__device__ __forceinline__ void for_units(uint32_t* ctr, uint32_t total, F&& unit) {
  uint32_t u = grab_unit(ctr);
  while (u < total) {
    uint32_t next = 0;
    if (lane_id() == 0) next = atomicAdd(ctr, 1u);
    unit(u);
    u = __builtin_amdgcn_readfirstlane(next);
  }
}

// flag bits and helpers of the one-launch placement (see lb_place_row)
constexpr uint64_t kLbAggregate = 1ull << 62, kLbPrefix = 2ull << 62, kLbAbort = 3ull << 62;
constexpr uint64_t kLbValue = (1ull << 62) - 1ull;

__device__ __forceinline__ void lb_store(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t lb_load(uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A single sign goes to memory for the caller only (later layers read it from the on-chip
// table): it bypasses the caches' keep-for-reuse policy, so that the text requested ahead stays cached.
__device__ __forceinline__ void store_single(uint64_t values, uint64_t g, uint64_t v) {
  __builtin_nontemporal_store(v, gptr<uint64_t>(values) + g);
}
// The same for any array entry that nothing on the device reads again (stream == true).
__device__ __forceinline__ void store_sign(G64 at, uint64_t v, bool stream) {
  if (stream) __builtin_nontemporal_store(v, at);
  else *at = v;
}

template <class Src>
struct Pass {
  const TileParams& P;
  const Sh& sh;
  const Src& src;
  uint32_t nb;        // records of this pass
  uint64_t g_first;   // batch-wide index of its first record
  uint32_t T, G;      // records per tile; operators a wavefront runs side by side
  uint32_t r, og;     // this lane's record and operator slot
  bool live;
  uint64_t g;
  uint32_t& malformed;
  bool& overflow;
  uint32_t lb_tile;   // tile number when counts are to be published (one-launch mode), else kNoRow
  bool need_table;    // the pass goes on to write: keep comma positions while counting
  bool split_all;     // filters and buckets with lists are counted a few lanes a field, like the hashes (counting launch)

  // This lane's place in a unit, worked out anew (and hidden from the optimiser's view of the
  // tile loop): otherwise every address that follows from it is computed once per kernel and
  // kept in a register of its own for good, and the hot loops run out of registers.
  __device__ __forceinline__ void refresh() {
    const uint32_t lane = lane_id();
    r = lane & (T - 1u);
    og = lane >> P.log2T;
    live = r < nb;
    g = g_first + r;
  }
  __device__ __forceinline__ uint32_t units_of(uint32_t list) const {
    return (sh.lbeg(list + 1) - sh.lbeg(list) + G - 1u) / G;
  }
  // the operator of this lane in unit u of a list, or null
  __device__ __forceinline__ const OpProg* op_of(uint32_t list, uint32_t u) const {
    const uint32_t lb = sh.lbeg(list), m = sh.lbeg(list + 1) - lb;
    const uint32_t i = u * G + og;
    return i < m ? &sh.prog[lb + i] : nullptr;
  }

  // ---- counts of the ragged root operators
  // Multi-valued hashes of staged records (the first P.n_mh entries of the ragged root list):
  // every wavefront takes part.  A few neighbouring lanes share one (operator, record) and
  // split the field at its commas: the item count, and the first item_cap comma positions
  // for the lanes that later hash the items.
  __device__ __forceinline__ void split_items() {
    const uint32_t tid = thread_id();
    const uint32_t np = P.n_mh * T;  // (operator, record slot) pairs
    uint32_t lg = 0;                 // log2 of the lanes per pair
    while (lg < 6u && (np << (lg + 1u)) <= kTileThreads) ++lg;
    const uint32_t j = tid & ((1u << lg) - 1u);
    for (uint32_t p0 = 0; p0 < np; p0 += kTileThreads >> lg) {
      const uint32_t pr = p0 + (tid >> lg);
      const uint32_t i = pr / T, rr = pr & (T - 1u);
      const bool act = pr < np && rr < nb;
      uint32_t s = 0, e = 0, row = 0;
      if (act) {
        const OpProg& d = sh.prog[sh.lbeg(TL_RAGROOT) + i];
        src.span(rr, d.field, s, e);
        row = d.rag_row;
      } else if (pr < np) {
        row = sh.prog[sh.lbeg(TL_RAGROOT) + i].rag_row;
      }
      uint16_t* tab = sh.ctab + pr * P.item_cap;
      const uint32_t cap = P.item_cap;
      const uint32_t commas = split_bytes(src.raw8, s, e, act, kCommas, lg, j, need_table ? cap : 0u, [&](uint32_t k, uint32_t pos) {
        tab[k] = (uint16_t)pos;
      });
      if (pr < np && j == 0) sh.cnt[row * T + rr] = act ? commas + 1u : 0u;  // items = commas + 1 (far below kMaxCount)
    }
  }
  // The other multi-valued root operators of staged records (filters and buckets: entries n_mh ..
  // n_split - 1 of the ragged root list) are counted the same way, a few lanes a field: a bucket
  // list has one sign per item; a filter tests the token that starts the field and the one after
  // every comma.  (A token is as long as the prefix or longer exactly when the prefix's bytes
  // follow its start and hold no comma: a prefix with a comma passes nothing, F_NEVER.)
  __device__ __forceinline__ void split_others() {
    const uint32_t tid = thread_id();
    const uint32_t np = (P.n_split - P.n_mh) * T;
    uint32_t lg = 0;
    while (lg < 6u && (np << (lg + 1u)) <= kTileThreads) ++lg;
    const uint32_t j = tid & ((1u << lg) - 1u);
    for (uint32_t p0 = 0; p0 < np; p0 += kTileThreads >> lg) {
      const uint32_t pr = p0 + (tid >> lg);
      const uint32_t i = pr / T, rr = pr & (T - 1u);
      const bool in = pr < np, act = in && rr < nb;
      const OpProg& d = sh.prog[sh.lbeg(TL_RAGROOT) + P.n_mh + (in ? i : 0u)];
      const bool filter = d.kind == OP_FILTER;
      uint32_t s = 0, e = 0;
      if (act) src.span(rr, d.field, s, e);
      uint32_t c;
      if (filter) {  // (uniform over the lanes of a field)
        const Prefix pre(sh.aux, d);
        uint32_t hits = (act && j == 0 && starts_with(src, s, e, pre)) ? 1u : 0u;
        split_bytes(src.raw8, s, e, act, kCommas, lg, j, ~0u, [&](uint32_t, uint32_t pos) {
          hits += starts_with(src, pos + 1u, e, pre) ? 1u : 0u;
        });
        for (uint32_t w = 1; w < (1u << lg); w <<= 1) hits += __shfl_xor(hits, (int)w, 64);
        c = (d.flags & F_NEVER) ? 0u : hits;
      } else {
        c = split_bytes(src.raw8, s, e, act, kCommas, lg, j, 0u, [](uint32_t, uint32_t) {}) + 1u;
      }
      if (in && j == 0) sh.cnt[d.rag_row * T + rr] = act ? c : 0u;
    }
  }
  // The single-valued filters and the n-grams (lists TL_RAGROOT and TL_NGRAM, taken as one), G
  // operators per unit; records read in place count all their ragged root operators here.
  __device__ __forceinline__ uint32_t count_skip() const { return !Src::kTable ? 0u : (split_all ? P.n_split : P.n_mh); }
  __device__ __forceinline__ uint32_t count_root_units() const {
    return (sh.lbeg(TL_RAGROOT + 1) - sh.lbeg(TL_RAGROOT) - count_skip() + G - 1u) / G;
  }
  __device__ __forceinline__ uint32_t count_units() const { return count_root_units() + units_of(TL_NGRAM); }
  __device__ __forceinline__ void count_unit(uint32_t u) {
    refresh();
    const uint32_t ur = count_root_units();
    const OpProg* d;
    uint32_t i = 0;  // position in the ragged root list
    if (u < ur) {
      const uint32_t lb = sh.lbeg(TL_RAGROOT), m = sh.lbeg(TL_RAGROOT + 1) - lb;
      i = count_skip() + u * G + og;
      d = i < m ? &sh.prog[lb + i] : nullptr;
    } else {
      d = op_of(TL_NGRAM, u - ur);
    }
    if (!d) return;
    uint32_t c = 0;
    if (live) {
      uint32_t s, e;
      src.span(r, d->field, s, e);
      if (d->kind == OP_NGRAM) {
        c = e - s >= d->aux_len ? e - s - d->aux_len + 1u : 0u;
      } else if (d->kind == OP_HASH && !need_table) {
        c = count_commas(src, s, e) + 1u;  // counting launch: nobody reads the comma table
      } else if (d->kind == OP_HASH) {
        // multi-valued hash: from comma to comma; the first item_cap positions are kept for the item lanes
        uint16_t* tab = sh.ctab + (i * T + r) * P.item_cap;
        uint32_t p = s;
        for (;;) {
          p = next_comma(src, p, e);
          if (p >= e) break;
          if (Src::kTable && c < P.item_cap) tab[c] = (uint16_t)p;
          ++c;
          ++p;
        }
        ++c;  // items = commas + 1
      } else {
        c = ragged_root_count(src, *d, sh.aux, s, e);
      }
    }
    if (c > kMaxCount) overflow = true;
    sh.cnt[d->rag_row * T + r] = c;
  }

  // Counts of the later layers follow from the inputs' counts, record by record and layer
  // by layer (the operators of one layer do not depend on each other): G operators per unit.
  __device__ __forceinline__ uint32_t derive_units(uint32_t layer) const {
    return (sh.rnr_head(layer - 1u) - sh.rnr_head(layer - 2u) + G - 1u) / G;
  }
  __device__ __forceinline__ void derive_unit(uint32_t layer, uint32_t u) {
    refresh();
    const uint32_t i = sh.rnr_head(layer - 2u) + u * G + og;
    if (i >= sh.rnr_head(layer - 1u)) return;
    const uint32_t header = 4u * ((P.n_layers + 3u) >> 2);
    const u32x4 d = *reinterpret_cast<const u32x4*>(sh.rnr + header + 4u * i);  // result row, a, b, cross or concat
    const uint64_t ca = (d.y >> 31) ? (d.y & 0x7fffffffu) : sh.cnt[d.y * T + r];
    const uint64_t cb = (d.z >> 31) ? (d.z & 0x7fffffffu) : sh.cnt[d.z * T + r];
    const uint64_t c = d.w == 0u ? ca * cb : ca + cb;
    if (c > kMaxCount) overflow = true;
    sh.cnt[d.x * T + r] = live ? (uint32_t)c : 0u;
  }
  // Counts become positions inside the tile: a prefix sum over the records of G rows at a time.
  // The ragged operators of the last layer (if it is not the first) hold the last rows, in the
  // order of their table entries: their counts are derived here, right before they are summed.
  __device__ __forceinline__ uint32_t last_layer_rows() const {
    return P.n_rnr ? sh.rnr_head(P.n_layers - 1u) - sh.rnr_head(P.n_layers - 2u) : 0u;
  }
  __device__ __forceinline__ uint32_t scan_units() const {
    const uint32_t nl = last_layer_rows();
    return (P.n_ragged - nl + G - 1u) / G + (nl + G - 1u) / G;
  }
  __device__ __forceinline__ void scan_unit(uint32_t u) {
    refresh();
    const uint32_t nl = last_layer_rows(), plain = P.n_ragged - nl, up = (plain + G - 1u) / G;
    uint32_t row, v = 0;
    bool ok;
    if (u < up) {
      row = u * G + og;
      ok = row < plain;
      if (ok) v = sh.cnt[row * T + r];
    } else {
      const uint32_t i = (u - up) * G + og;
      row = plain + i;
      ok = i < nl;
      if (ok) {
        const uint32_t header = 4u * ((P.n_layers + 3u) >> 2);
        const u32x4 d = *reinterpret_cast<const u32x4*>(sh.rnr + header + 4u * (sh.rnr_head(P.n_layers - 2u) + i));
        const uint64_t ca = (d.y >> 31) ? (d.y & 0x7fffffffu) : sh.cnt[d.y * T + r];
        const uint64_t cb = (d.z >> 31) ? (d.z & 0x7fffffffu) : sh.cnt[d.z * T + r];
        const uint64_t c = d.w == 0u ? ca * cb : ca + cb;
        if (c > kMaxCount) overflow = true;
        v = live && c <= kMaxCount ? (uint32_t)c : 0u;
        sh.cnt[row * T + r] = v;
      }
    }
    const uint32_t incl = group_incl_scan(v, T);
    if (ok) {
      const uint32_t before = sh.run[row];
      sh.start[row * T + r] = before + incl - v;
      if (r == T - 1u) {
        sh.run[row] = before + incl;
        sh.tot[row] = incl;
        if (lb_tile != kNoRow && !row_follows(P, sh, row))  // one-launch mode: later tiles may need it at once
          lb_store(P.lb_state + (uint64_t)row * P.n_tiles + lb_tile, kLbAggregate | incl);
      }
    }
  }

  // ---- layer 1
  // (a unit is 2 G operators, each lane taking two of them one after the other: half the hand-outs and set-ups)
  static constexpr uint32_t kHashPairs = 1;  // pairs of operators a lane hashes per unit (two pairs measured 1.6 % slower: fewer, longer units balance worse)
  __device__ __forceinline__ uint32_t hash1_units() const {
    return (sh.lbeg(TL_HASH1 + 1) - sh.lbeg(TL_HASH1) + 2u * kHashPairs * G - 1u) / (2u * kHashPairs * G);
  }
  __device__ __forceinline__ void hash1_unit(uint32_t u) {
    refresh();
    if (!live) return;
#pragma unroll
    for (uint32_t pair = 0; pair < kHashPairs; ++pair) hash1_pair(u * kHashPairs + pair);
  }
  __device__ __forceinline__ void hash1_pair(uint32_t u) {
    const uint32_t lb = sh.lbeg(TL_HASH1), m = sh.lbeg(TL_HASH1 + 1) - lb;
    // both operators' programs and fields are looked up before either is hashed: the look-ups
    // (program, then field table) are waited for once, not once per operator
    const uint32_t i0 = 2u * u * G + og, i1 = i0 + G;
    const bool two = i1 < m;
    if (i0 >= m) return;
    const OpProg& d0 = sh.prog[lb + i0];
    const OpProg& d1 = sh.prog[lb + (two ? i1 : i0)];
    uint32_t s0, e0, s1, e1;
    src.span(r, d0.field, s0, e0);
    src.span(r, d1.field, s1, e1);
    const uint64_t v0 = hash_span(src, s0, e0, d0.key);
    store_single(d0.values, g, v0);
    if (d0.stage != kNoRow) sh.stage[d0.stage * T + r] = v0;
    if (!two) return;
    const uint64_t v1 = hash_span(src, s1, e1, d1.key);
    store_single(d1.values, g, v1);
    if (d1.stage != kNoRow) sh.stage[d1.stage * T + r] = v1;
  }
  __device__ __forceinline__ void bucket1_unit(uint32_t u) {
    refresh();
    const OpProg* d = op_of(TL_BUCKET1, u);
    if (!d || !live) return;
    uint32_t s, e;
    src.span(r, d->field, s, e);
    bool bad;
    const int64_t x = parse_micro(src, s, e, bad);
    malformed += bad ? 1u : 0u;
    const uint64_t v = bucket_of(x, d->key, sh.aux, d->aux_off, d->aux_len);
    store_single(d->values, g, v);
    if (d->stage != kNoRow) sh.stage[d->stage * T + r] = v;
  }
  // where this lane's list of a ragged operator starts; writes its offsets entry
  __device__ __forceinline__ uint64_t place(const OpProg& d, uint32_t rr, uint64_t gg) const {
    const uint64_t first = sh.base[d.rag_row] + sh.start[d.rag_row * T + rr];
    if (d.flags & F_EMIT) {
      G64 off = gptr<uint64_t>(d.offsets);
      __builtin_nontemporal_store(first, off + gg);
      if (gg + 1 == P.n_records) off[gg + 1] = first + sh.cnt[d.rag_row * T + rr];
    }
    return first;
  }
  // the other ragged root operators (filters, multi-valued buckets): a lane writes its record's list
  __device__ __forceinline__ uint32_t other_units() const {
    return (sh.lbeg(TL_RAGROOT + 1) - sh.lbeg(TL_RAGROOT) - P.n_mh + G - 1u) / G;
  }
  __device__ __forceinline__ void other_unit(uint32_t u) {
    refresh();
    const uint32_t lb = sh.lbeg(TL_RAGROOT) + P.n_mh, m = sh.lbeg(TL_RAGROOT + 1) - lb;
    const uint32_t i = u * G + og;
    const OpProg* d = i < m ? &sh.prog[lb + i] : nullptr;
    if (!d || !live) return;
    const uint64_t first = place(*d, r, g);
    uint32_t s, e;
    src.span(r, d->field, s, e);
    ragged_root_emit(src, *d, sh.aux, s, e, gptr<uint64_t>(d->values) + first, malformed);
  }
  // Multi-valued hashes (the first P.n_mh entries of the ragged root list): lanes
  // are items.  All items of the pass, operator after operator and record after
  // record, form one index space; a lane finds its operator and record by two
  // small searches, its item's bounds in the comma table, and writes the sign to
  // the item's own position: neighbouring lanes write neighbouring signs.
  __device__ __forceinline__ void item_offsets() {  // one wavefront, after the positions are known
    const uint32_t lane = lane_id();
    uint32_t carry = 0;
    for (uint32_t i0 = 0; i0 < P.n_mh; i0 += 64u) {
      const uint32_t i = i0 + lane;
      uint32_t v = 0;
      if (i < P.n_mh) v = sh.tot[sh.prog[sh.lbeg(TL_RAGROOT) + i].rag_row];
      uint32_t incl = v;
      for (uint32_t d = 1; d < 64u; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
      }
      if (i < P.n_mh) sh.ioff[i] = carry + incl - v;
      carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) sh.ioff[P.n_mh] = carry;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  }
  __device__ __forceinline__ uint32_t item_units() const { return (sh.ioff[P.n_mh] + 63u) >> 6; }
  __device__ __forceinline__ void item_unit(uint32_t u) {
    const uint32_t q = u * 64u + lane_id();
    if (q >= sh.ioff[P.n_mh]) return;
    // operator: the last one whose first item is <= q
    uint32_t lo = 0, hi = P.n_mh - 1u;
    while (lo < hi) {
      const uint32_t mid = (lo + hi + 1u) >> 1;
      if (sh.ioff[mid] <= q) lo = mid; else hi = mid - 1u;
    }
    const uint32_t i = lo;
    const OpProg& d = sh.prog[sh.lbeg(TL_RAGROOT) + i];
    const uint32_t row = d.rag_row;
    const uint32_t before = sh.run[row] - sh.tot[row];     // signs of the tile's earlier passes
    const uint32_t pos = before + (q - sh.ioff[i]);         // the item's position inside the tile
    // record: the last one whose first position is <= pos (every record has at least one item)
    const uint32_t* st = sh.start + row * T;
    lo = 0; hi = nb - 1u;
    while (lo < hi) {
      const uint32_t mid = (lo + hi + 1u) >> 1;
      if (st[mid] <= pos) lo = mid; else hi = mid - 1u;
    }
    const uint32_t rr = lo, j = pos - st[rr], cnt = sh.cnt[row * T + rr];
    uint32_t s, e;
    src.span(rr, d.field, s, e);
    const uint16_t* tab = sh.ctab + (i * T + rr) * P.item_cap;
    const uint32_t cap = Src::kTable ? P.item_cap : 0u;
    uint32_t is, ie;
    if (j == 0) {
      is = s;
    } else if (j <= cap) {
      is = (uint32_t)tab[j - 1u] + 1u;
    } else {  // beyond the table: walk on from its last comma
      is = cap ? (uint32_t)tab[cap - 1u] + 1u : s;
      for (uint32_t c = cap; c < j; ++c) is = next_comma(src, is, e) + 1u;
    }
    if (j + 1u == cnt) ie = e;
    else if (j < cap) ie = tab[j];
    else ie = next_comma(src, is, e);
    const uint64_t first = sh.base[row] + pos;
    if (j == 0 && (d.flags & F_EMIT)) {
      G64 off = gptr<uint64_t>(d.offsets);
      const uint64_t gg = g_first + rr;
      __builtin_nontemporal_store(first, off + gg);
      if (gg + 1 == P.n_records) off[gg + 1] = first + cnt;
    }
    const uint64_t v = hash_span(src, is, ie, d.key);
    store_sign(gptr<uint64_t>(d.values) + first, v, d.flags & F_STREAM);
    // crosses of this hash with a single sign: one sign per item, in the items' order
    const uint32_t* fused = sh.rnr + 4u * ((P.n_layers + 3u) >> 2) + 4u * P.n_rnr + d.a;
    for (uint32_t k = 0; k < d.b; ++k) {
      const OpProg& c = sh.prog[fused[k]];
      const uint64_t other = sh.stage[c.aux_off * T + rr];
      const uint64_t at = sh.base[c.rag_row] + sh.start[c.rag_row * T + rr] + j;
      if (j == 0 && (c.flags & F_EMIT)) {
        G64 off = gptr<uint64_t>(c.offsets);
        const uint64_t gg = g_first + rr;
        __builtin_nontemporal_store(at, off + gg);
        if (gg + 1 == P.n_records) off[gg + 1] = at + cnt;
      }
      store_sign(gptr<uint64_t>(c.values) + at, c.aux_len ? mix64(mix64(v + c.key) + other) : mix64(mix64(other + c.key) + v),
                 c.flags & F_STREAM);
    }
  }

  // n-grams: the lanes of a wavefront run over the grams of one record; unit = (operator, record)
  __device__ __forceinline__ uint32_t ngram_units() const {
    return (sh.lbeg(TL_NGRAM + 1) - sh.lbeg(TL_NGRAM)) * nb;
  }
  __device__ __forceinline__ void ngram_unit(uint32_t u) {
    const uint32_t lane = lane_id();
    const OpProg& d = sh.prog[sh.lbeg(TL_NGRAM) + u / nb];
    const uint32_t rr = u % nb;
    uint32_t s, e;
    src.span(rr, d.field, s, e);
    const uint32_t ng = sh.cnt[d.rag_row * T + rr], n = d.aux_len;
    uint64_t first = 0;
    if (lane == 0) first = place(d, rr, g_first + rr);
    first = __shfl(first, 0, 64);
    G64 vals = gptr<uint64_t>(d.values) + first;
    const uint64_t key = d.key;
    for (uint32_t q = lane; q < ng; q += 64) vals[q] = hash_span(src, s + q, s + q + n, key);
  }

  // A 64-bit literal of generated code, handed over in scalar registers at the place of its use (otherwise
  // the compiler collects every operator's key in vector registers ahead of the tile loop, and spills them).
  static __device__ __forceinline__ uint64_t here(uint64_t k) {
    uint32_t lo = (uint32_t)k, hi = (uint32_t)(k >> 32);
    asm volatile("" : "+s"(lo), "+s"(hi));
    return ((uint64_t)hi << 32) | lo;
  }
  // ---- one operator on the (up to 64) records of a tile, one record per lane
  // For tiles of 64 records a wavefront runs one single-sign operator at a time, and what the
  // operator is (field, key, table rows) is the same in every lane.  In a kernel generated for
  // the plan these are literals of straight-line code, one piece per operator (the meta-kernel
  // of Section 4, "Inner-GPU operator launching": each operator a device function, called one
  // after the other); `op` is the operator's number, under which its array's address lies in the
  // per-call program table (read through the scalar unit).  Staged records only.
  // where a single sign of operator `op` goes: to the caller's array (streamed, nothing on the device
  // reads it again) and, if a later operator reads it, to the on-chip table
  __device__ __forceinline__ void lane_put(uint32_t lane, uint64_t values, uint32_t stage, uint64_t v) const {
    __builtin_nontemporal_store(v, gptr<uint64_t>(values) + g_first + lane);
    if (stage != kNoRow) sh.stage[stage * 64u + lane] = v;
  }
  // the address of operator op's array, from the per-call program table through the scalar unit
  // (generated code: the same address in every lane)
  __device__ __forceinline__ uint64_t values_of(uint32_t op) const { return cptr(P.prog)[op].values; }
  __device__ __forceinline__ void lane_hash1(uint32_t field, uint64_t key, uint64_t values, uint32_t stage) const {
    const uint32_t lane = lane_id();
    if (lane >= nb) return;
    uint32_t s, e;
    src.span(lane, field, s, e);
    lane_put(lane, values, stage, hash_span(src, s, e, key));
  }
  __device__ __forceinline__ void lane_bucket1(uint32_t field, uint64_t key, uint32_t aux_off, uint32_t n_bounds, uint64_t values,
                                               uint32_t stage) {
    const uint32_t lane = lane_id();
    if (lane >= nb) return;
    uint32_t s, e;
    src.span(lane, field, s, e);
    bool bad;
    const int64_t v = parse_micro(src, s, e, bad);
    malformed += bad ? 1u : 0u;
    lane_put(lane, values, stage, bucket_of(v, key, sh.aux, aux_off, n_bounds));
  }
  __device__ __forceinline__ void lane_x11(uint32_t stage_a, uint32_t stage_b, uint64_t key, uint64_t values, uint32_t stage) const {
    const uint32_t lane = lane_id();
    if (lane >= nb) return;
    const uint64_t a = sh.stage[stage_a * 64u + lane], b = sh.stage[stage_b * 64u + lane];
    lane_put(lane, values, stage, mix64(mix64(a + key) + b));
  }
#if FBX_LANE_OPS == 2
  // generated: one case per single-valued bucket, then one per single-valued hash, in the order of
  // the work lists; per later layer one case per cross of two single signs
  __device__ __forceinline__ void lane_l1_unit(uint32_t u) {
    switch (u) { FBX_GEN_L1 }
  }
  __device__ __forceinline__ void lane_x11_unit(uint32_t layer, uint32_t u) {
    switch (layer) { FBX_GEN_X11 }
  }
#else
  // the same bodies, the operator's numbers read from the program table in LDS (one small piece of code for all)
  __device__ __forceinline__ void lane_l1_unit(uint32_t u) {
    const uint32_t ub = sh.lbeg(TL_BUCKET1 + 1) - sh.lbeg(TL_BUCKET1);
    if (u < ub) {
      const OpProg& d = sh.prog[sh.lbeg(TL_BUCKET1) + u];
      lane_bucket1(d.field, d.key, d.aux_off, d.aux_len, d.values, d.stage);
    } else {
      const OpProg& d = sh.prog[sh.lbeg(TL_HASH1) + (u - ub)];
      lane_hash1(d.field, d.key, d.values, d.stage);
    }
  }
  __device__ __forceinline__ void lane_x11_unit(uint32_t layer, uint32_t u) {
    const OpProg& d = sh.prog[sh.lbeg(TL_LAYER + 2u * (layer - 2u)) + u];
    lane_x11(d.aux_off, d.aux_len, d.key, d.values, d.stage);
  }
#endif

  // ---- later layers
  // crosses of two single signs, both on chip
  static constexpr uint32_t kCrossesPerLane = 2;  // (two a lane: half the hand-outs; measured 0.7 % on the largest workload)
  __device__ __forceinline__ uint32_t x11_units(uint32_t layer) const {
    const uint32_t list = TL_LAYER + 2u * (layer - 2u);
    return (sh.lbeg(list + 1) - sh.lbeg(list) + kCrossesPerLane * G - 1u) / (kCrossesPerLane * G);
  }
  __device__ __forceinline__ void x11_unit(uint32_t layer, uint32_t u) {
    refresh();
    if (!live) return;
    const uint32_t list = TL_LAYER + 2u * (layer - 2u);
    const uint32_t lb = sh.lbeg(list), m = sh.lbeg(list + 1) - lb;
    // (a cross never reads a cross of its own layer: the crosses of a unit are independent, their inputs are requested together)
    const OpProg* d[kCrossesPerLane];
    uint64_t a[kCrossesPerLane], b[kCrossesPerLane];
#pragma unroll
    for (uint32_t k = 0; k < kCrossesPerLane; ++k) {
      const uint32_t i = (u * kCrossesPerLane + k) * G + og;
      d[k] = i < m ? &sh.prog[lb + i] : nullptr;
    }
#pragma unroll
    for (uint32_t k = 0; k < kCrossesPerLane; ++k)
      if (d[k]) { a[k] = sh.stage[d[k]->aux_off * T + r]; b[k] = sh.stage[d[k]->aux_len * T + r]; }
#pragma unroll
    for (uint32_t k = 0; k < kCrossesPerLane; ++k) {
      if (!d[k]) continue;
      const uint64_t v = mix64(mix64(a[k] + d[k]->key) + b[k]);
      store_single(d[k]->values, g, v);
      if (d[k]->stage != kNoRow) sh.stage[d[k]->stage * T + r] = v;
    }
  }
  // Every other cross or concat: lanes are output signs.  The signs that the list operators of
  // one layer produce in this pass, operator after operator and record after record, form one
  // index space; a unit is 64 consecutive ones, whichever operators they belong to, so that
  // operators with few signs share wavefronts.  A lane finds its operator by a search over the
  // operators' first signs (gen_offsets), its record by a search over the records' first
  // positions; its place in the record's list tells which input signs it combines, and
  // neighbouring lanes write neighbouring signs.  Units before those hand the offsets entries of
  // the ragged operators to lanes, one (operator, record) each.
  __device__ __forceinline__ uint32_t gen_total(const OpProg& d) const { return d.arity ? d.arity * nb : sh.tot[d.rag_row]; }
  __device__ __forceinline__ uint32_t gen_list(uint32_t layer) const { return TL_LAYER + 2u * (layer - 2u) + 1u; }
  // one wavefront, after the positions are known: where every list operator's signs start
  __device__ __forceinline__ void gen_offsets() {
    const uint32_t lane = lane_id();
    for (uint32_t layer = 2; layer <= P.n_layers; ++layer) {
      const uint32_t lb = sh.lbeg(gen_list(layer)), m = sh.lbeg(gen_list(layer) + 1u) - lb;
      uint32_t carry = 0;
      for (uint32_t i0 = 0; i0 < m; i0 += 64u) {
        const uint32_t i = i0 + lane;
        const uint32_t v = i < m ? gen_total(sh.prog[lb + i]) : 0u;
        const uint32_t incl = group_prefix(v, 6u, lane);
        if (i < m) sh.gfirst[lb + i] = carry + incl - v;
        carry += __shfl(incl, 63, 64);
      }
      if (lane == 0) sh.gtot[layer] = carry;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  }
  // sign x of record rr of an earlier operator (single signs from the on-chip table, lists
  // from the arrays this workgroup wrote before the layer barrier)
  __device__ __forceinline__ uint64_t input_sign(const OpProg& d, uint32_t rr, uint32_t x) const {
    if (d.arity == 1u && d.stage != kNoRow) return sh.stage[d.stage * T + rr];
    const uint64_t at = d.arity ? (g_first + rr) * d.arity : sh.base[d.rag_row] + sh.start[d.rag_row * T + rr];
    return gptr<const uint64_t>(d.values)[at + x];
  }
  __device__ __forceinline__ uint32_t gen_place_units(uint32_t layer) const {
    return (sh.lbeg(gen_list(layer) + 1u) - sh.lbeg(gen_list(layer)) + G - 1u) / G;
  }
  __device__ __forceinline__ uint32_t gen_units(uint32_t layer) const { return gen_place_units(layer) + ((sh.gtot[layer] + 63u) >> 6); }
  __device__ __forceinline__ void gen_unit(uint32_t layer, uint32_t u) {
    const uint32_t lb = sh.lbeg(gen_list(layer)), m = sh.lbeg(gen_list(layer) + 1u) - lb;
    const uint32_t up = gen_place_units(layer);
    if (u < up) {  // the offsets entries: a lane takes one record of one operator
      refresh();
      const uint32_t i = u * G + og;
      if (i < m && live) {
        const OpProg& d = sh.prog[lb + i];
        if (!d.arity) place(d, r, g);
      }
      return;
    }
    const uint32_t q = (u - up) * 64u + lane_id();
    if (q >= sh.gtot[layer]) return;
    // operator: the last one whose first sign is <= q (operators without signs in this pass share
    // their first sign with the one after them and are passed over)
    uint32_t lo = 0, hi = m - 1u;
    while (lo < hi) {
      const uint32_t mid = (lo + hi + 1u) >> 1;
      if (sh.gfirst[lb + mid] <= q) lo = mid; else hi = mid - 1u;
    }
    const OpProg& d = sh.prog[lb + lo];
    const uint32_t qq = q - sh.gfirst[lb + lo];  // the sign's number among the operator's signs of this pass
    const uint32_t row = d.rag_row;
    uint32_t rr, j;
    uint64_t at;  // where the sign goes
    if (d.arity) {
      rr = qq / d.arity;
      j = qq - rr * d.arity;
      at = (g_first + rr) * d.arity + j;
    } else {
      const uint32_t pos = sh.run[row] - sh.tot[row] + qq;  // position inside the tile (earlier passes come first)
      const uint32_t* st = sh.start + row * T;
      uint32_t l2 = 0, h2 = nb - 1u;  // the last record whose first position is <= pos (it is the one that has the sign)
      while (l2 < h2) {
        const uint32_t mid = (l2 + h2 + 1u) >> 1;
        if (st[mid] <= pos) l2 = mid; else h2 = mid - 1u;
      }
      rr = l2;
      j = pos - st[rr];
      at = sh.base[row] + pos;
    }
    const OpProg& da = sh.prog[d.a];
    const OpProg& db = sh.prog[d.b];
    const uint32_t na = da.arity ? da.arity : sh.cnt[da.rag_row * T + rr];
    const uint32_t nbv = db.arity ? db.arity : sh.cnt[db.rag_row * T + rr];
    uint64_t v;
    if (d.kind == OP_CROSS) {  // A outer, B inner
      const uint32_t x = j / nbv, y = j - x * nbv;
      v = mix64(mix64(input_sign(da, rr, x) + d.key) + input_sign(db, rr, y));
    } else {
      v = j < na ? input_sign(da, rr, j) : input_sign(db, rr, j - na);
    }
    store_sign(gptr<uint64_t>(d.values) + at, v, d.flags & F_STREAM);
  }
};

// ---- ordered placement without a counting launch (MODE 2)
// Every (ragged operator, tile) has one 64-bit word: two flag bits and a number
// of signs.  A tile publishes its count (AGGREGATE) as soon as it knows it.  To
// find its base it then reads the words of the 64 tiles before it at once, one per
// lane: the nearest word that already holds "signs up to and including this tile"
// (PREFIX) plus the counts of the tiles in between is the answer; if all 64 are
// counts the window moves on.  The tile finally publishes its own PREFIX, so the
// distance to the nearest PREFIX stays a small fraction of the tiles in flight.
// Workgroups take every W-th tile, so a tile only ever waits for tiles that
// other running workgroups are counting right now; waits that still exceed
// P.spin_limit polls are given up and reported.  ABORT marks a tile that cannot be
// placed (bad offsets, text larger than the LDS section, array capacity
// exceeded); it spreads to all later tiles, which then write nothing, and the
// call is repeated with a counting launch.

// Marks the tile as not placeable for every ragged operator.
__device__ __forceinline__ void lb_abort_tile(const TileParams& P, uint32_t tile) {
  for (uint32_t row = threadIdx.x; row < P.n_ragged; row += kTileThreads)
    lb_store(P.lb_state + (uint64_t)row * P.n_tiles + tile, kLbAbort);
}

// The words of the 64 tiles below `upper` of one ragged operator, lane 0 the nearest;
// in front of tile 0 lies a prefix of zero.
__device__ __forceinline__ uint64_t lb_window(const TileParams& P, uint32_t row, uint32_t upper) {
  const uint32_t lane = lane_id();
  return upper > lane ? lb_load(P.lb_state + (uint64_t)row * P.n_tiles + (upper - 1u - lane)) : kLbPrefix;
}

// One wavefront finds the base of one ragged operator for this tile (whose count is
// already published).  `v` is the window right below the tile, requested by the caller
// (who requests those of several operators at once, so that their latencies overlap).
// Returns false (in every lane) when the tile must not be written.
__device__ __forceinline__ bool lb_place_row(const TileParams& P, const Sh& sh, uint32_t tile, uint32_t row, uint64_t v) {
  const uint32_t lane = lane_id();
  uint64_t* st = P.lb_state + (uint64_t)row * P.n_tiles;
  const uint64_t agg = sh.tot[row];
  uint64_t excl = 0;
  bool abort = false;
  uint32_t upper = tile, spins = 0;
  FBX_TALLY(15, 1);  // (tuning builds: placements, windows read, polls of an unfinished tile)
  for (;; v = lb_window(P, row, upper)) {
    FBX_TALLY(13, 1);
    // the wait is bounded: after P.spin_limit polls that found an unfinished tile it is given up
    // (a limit of zero gives up before the first look: how a test forces the condition from the host)
    if (spins >= P.spin_limit) {
      if (lane == 0) atomicOr(&P.ctrl->err, (uint32_t)CE_STALL);
      abort = true;
      break;
    }
    const uint64_t flag = v & ~kLbValue;
    const uint64_t stops = __ballot(flag == kLbPrefix || flag == kLbAbort);
    const uint32_t stop = stops ? (uint32_t)__ffsll((unsigned long long)stops) - 1u : 64u;
    const uint64_t below = stop == 64u ? ~0ull : ((1ull << stop) - 1ull);
    if (__ballot(flag == 0ull) & below) {  // a tile in between has not counted yet
      FBX_TALLY(14, 1);
      ++spins;
      __builtin_amdgcn_s_sleep(4);
      continue;
    }
    uint64_t part = (lane < stop || (lane == stop && flag == kLbPrefix)) ? (v & kLbValue) : 0ull;
    for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
    excl += part;
    if (stop < 64u) {
      abort = __shfl(flag, (int)stop, 64) == kLbAbort;
      break;
    }
    upper -= 64u;  // all counts: look further back (upper >= 64 here, else lane `upper` had stopped the window)
    spins = 0;
  }
  bool small = !abort && excl + agg > sh.cap[row];  // an array was sized too small: nothing may be written
  if (P.n_alias && !abort) {
    // the rows that follow this one: scale * (its signs before the tile) + add * (records before the tile)
    for (uint32_t c0 = 0; c0 < P.n_ragged; c0 += 64u) {
      const uint32_t c = c0 + lane;
      if (c >= P.n_ragged) continue;
      const uint32_t* a = sh.rnr + P.alias_at + 3u * c;
      if (a[0] != row) continue;
      const uint64_t before = (uint64_t)a[1] * excl + (uint64_t)a[2] * ((uint64_t)tile << P.log2T);
      if (__umul64hi((uint64_t)a[1], excl) != 0ull || before + sh.tot[c] > sh.cap[c]) {
        small = true;
      } else {
        sh.base[c] = before;
        if (tile + 1u == P.n_tiles) gptr(P.row_actual)[c] = before + sh.tot[c];
      }
    }
  }
  if (__ballot(small)) {
    if (lane == 0) atomicOr(&P.ctrl->err, (uint32_t)CE_SPEC);
    abort = true;
  }
  if (lane == 0) {
    lb_store(st + tile, abort ? kLbAbort : (kLbPrefix | (excl + agg)));
    sh.base[row] = excl;
    if (tile + 1u == P.n_tiles) gptr(P.row_actual)[row] = excl + agg;
  }
  return !abort;
}

// Runs every layer on the nb records of one pass.  WRITE = false stops after the
// counts.  hook() is called by every lane right after barriers (the caller
// advances the next tile's loads there).
template <int MODE, class Src, class Hook>
__device__ __forceinline__ void run_pass(const TileParams& P, const Sh& sh, const Src& src, uint32_t nb, uint64_t g_first,
                                         uint32_t tile, uint32_t& malformed, bool& overflow, Hook&& hook) {
  constexpr bool WRITE = MODE != 0;
  const uint32_t tid = thread_id(), lane = tid & 63u, wave = tid >> 6;
  const uint32_t T = 1u << P.log2T;
  Pass<Src> ps{P, sh, src, nb, g_first, T, 64u >> P.log2T, lane & (T - 1u), lane >> P.log2T, false, 0, malformed, overflow, MODE == 2 ? tile : kNoRow, WRITE, MODE == 0};
  ps.live = ps.r < nb;
  ps.g = g_first + ps.r;
  // the single-valued hashes and buckets of layer 1 fill whatever phase has idle wavefronts
  // tiles of 64 staged records in a kernel compiled for the plan: one single-sign operator a unit, one record a lane
  constexpr bool kGen = FBX_LANE_OPS != 0 && Src::kTable;
  const uint32_t ub = WRITE ? ps.units_of(TL_BUCKET1) : 0u;
  const uint32_t uh = !WRITE ? 0u : (kGen ? sh.lbeg(TL_HASH1 + 1) - sh.lbeg(TL_HASH1) : ps.hash1_units());
  auto l1_unit = [&](uint32_t u) {
    if (FBX_SKIP(1u)) return;
    if constexpr (kGen) { ps.lane_l1_unit(u); return; }
    if (u < ub) ps.bucket1_unit(u); else ps.hash1_unit(u - ub);  // (the longer units first: a shorter tail)
  };
  // (the code generated for a plan's operators is large: it stays in one place, the loop of phase C, and
  // wavefronts that find no counting unit left then just wait)
  auto fill_one = [&]() -> bool {
    if constexpr (kGen) return false;
    const uint32_t u = grab_unit(&s_ctr[0]);
    if (u >= uh + ub) return false;
    if (FBX_SKIP(1u)) return true;
    if (u < ub) ps.bucket1_unit(u); else ps.hash1_unit(u - ub);  // (the longer units first: a shorter tail)
    return true;
  };

  // A phase whose few long units would leave most wavefronts idle: wavefronts that
  // find no unit left hash single-valued fields until the last unit is done.
  auto critical_phase = [&](uint32_t total, uint32_t* ctr, uint32_t* done, auto&& unit) {
    for (uint32_t u = grab_unit(ctr); u < total; u = grab_unit(ctr)) {
      unit(u);
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
      if (lane == 0) atomicAdd(done, 1u);
    }
    if (WRITE) {
      while (*reinterpret_cast<volatile uint32_t*>(done) < total && fill_one()) {}
    }
    __syncthreads();
  };

  // ---- phase A: counts of the ragged root operators
  bool absurd = false;
  if constexpr (Src::kTable) {
    if (P.n_mh) ps.split_items();
    if (P.n_mh && FBX_SKIP(0x200u)) {  // (tuning builds: once more, to weigh it)
      __syncthreads();
      ps.split_items();
    }
    // (the counting launch only: a launch that writes has single-valued fields to hash while a few
    // wavefronts count these operators unit by unit, below)
    if (MODE == 0 && P.n_split > P.n_mh) ps.split_others();
  }
  if (P.n_ragged) critical_phase(ps.count_units(), &s_ctr[1], &s_done, [&](uint32_t u) { ps.count_unit(u); });
  else __syncthreads();
  if (P.n_ragged && FBX_SKIP(0x800u)) {  // (tuning builds: the counting units once more, to weigh them)
    for (uint32_t u = wave; u < ps.count_units(); u += kWaves) ps.count_unit(u);
    __syncthreads();
  }
  FBX_MARK(4);
  hook();
  // ---- phase B: the counts of later layers, layer by layer
  if (P.n_rnr) {
    // (short: the wavefronts just share the units out; the last layer's counts are left to the next phase)
    for (uint32_t layer = 2; layer < P.n_layers; ++layer) {
      const uint32_t ud = ps.derive_units(layer);
      for (uint32_t u = wave; u < ud; u += kWaves) ps.derive_unit(layer, u);
      __syncthreads();
      hook();
    }
    FBX_MARK(5);
  }
  // ---- phase B2: counts become positions
  if (P.n_ragged) {
    const uint32_t us = ps.scan_units();
    for (uint32_t u = wave; u < us; u += kWaves) ps.scan_unit(u);
    if (MODE >= 2 && overflow) s_absurd = 1u;  // (rare: a plain flag is cheaper than a vote in every tile)
    __syncthreads();
    if (MODE >= 2) absurd = s_absurd != 0u;
    FBX_MARK(6);
    hook();
  }
  if (MODE >= 2 && absurd) {  // absurd counts: nothing of this tile may be placed (whatever it published is overwritten)
    if (MODE == 2) lb_abort_tile(P, tile);
    return;
  }
  if (!WRITE) return;

  // ---- phase C: the rest of layer 1's single signs; one wavefront first lays out the item
  // index space of the multi-valued hashes (needed after at least one more barrier)
  if (P.n_mh && wave == kWaves - 1) ps.item_offsets();
  if (P.n_gen && wave == kWaves - 2) ps.gen_offsets();  // (likewise: where the list operators' signs start)
  // Arrival order (Section 5, Algorithm 1 with the tile's share of a ragged operator as the block): one
  // atomic add per (operator, tile) on the operator's running total; tiles land in the order in which
  // they get here.  Where the tile's share ends goes into the table that the look-back words occupy in
  // mode 2: a record's list ends where the next record's starts, except for a tile's last record.
  auto place_by_arrival = [&]() {  // one wavefront
    bool small = false;
    for (uint32_t row = lane; row < P.n_ragged; row += 64u) {
      const uint64_t n = sh.tot[row];
      const uint64_t at = atomicAdd(reinterpret_cast<unsigned long long*>(P.row_actual) + row, (unsigned long long)n);
      if (at + n > sh.cap[row]) {
        small = true;  // the array was sized too small: nothing may be written
      } else {
        sh.base[row] = at;
        gptr(P.lb_state)[(uint64_t)row * P.n_tiles + tile] = at + n;
      }
    }
    if (__ballot(small) && lane == 0) {
      atomicOr(&P.ctrl->err, (uint32_t)CE_SPEC);
      s_good = 0u;
    }
  };
  // Launches that know a tile's bases early (from the scan over tiles, or by arrival): the ragged root
  // operators share a hand-out with the last layer of single crosses, long units first.  (The last
  // layer: a cross computed along with a multi-valued hash's items reads a single sign of any earlier
  // layer, which must be in place; nothing on the chip reads the last layer's single signs.)
  constexpr bool kEarlyBases = MODE == 1 || MODE == 3;
  if (kEarlyBases && MODE == 3 && P.n_ragged && wave == 0) place_by_arrival();
  auto ragged_root_units = [&]() -> uint32_t {
    return (P.n_mh ? ps.item_units() : 0u) + ps.other_units() + ps.ngram_units();
  };
  auto ragged_root_unit = [&](uint32_t u) {
    if (FBX_SKIP(4u)) return;
    const uint32_t um = P.n_mh ? ps.item_units() : 0u, uo = ps.other_units();
    if (u < uo) ps.other_unit(u);
    else if (u < uo + um) ps.item_unit(u - uo);
    else ps.ngram_unit(u - uo - um);
  };
  bool ragged_roots_done = false;
  for_units(&s_ctr[0], uh + ub, l1_unit);
  FBX_MARK(7);
  // One-launch mode: the words of the tiles before this one (for the wavefront's first ragged
  // operator) are requested now, so that they arrive while the single crosses run.
  uint64_t early = kLbPrefix;
  if (MODE == 2 && wave < P.n_ragged && !row_follows(P, sh, wave)) early = lb_window(P, wave, tile);
  // ---- the single crosses of every later layer: they only read signs kept on chip
  for (uint32_t layer = 2; layer <= P.n_layers; ++layer) {
    __syncthreads();  // the layer barrier: every sign this layer reads is in place
    hook();
    uint32_t* ctr = &s_ctr[4u + (layer & 1u)];
    if (tid == 0) s_ctr[4u + ((layer + 1u) & 1u)] = 0;  // the next layer's counter (idle since the barrier before this one)
    const uint32_t ux = kGen ? ps.units_of(TL_LAYER + 2u * (layer - 2u)) : ps.x11_units(layer);
    uint32_t ur = 0;
    if (kEarlyBases && layer == P.n_layers && P.n_ragged) {
      if (MODE == 3 && !s_good) return;  // the call falls back: leave the arrays alone
      ur = ragged_root_units();
      ragged_roots_done = true;
    }
    for_units(ur ? &s_ctr[3] : ctr, ur + ux, [&](uint32_t u) {
      if (u < ur) { ragged_root_unit(u); return; }
      if (FBX_SKIP(2u)) return;
      if constexpr (kGen) { ps.lane_x11_unit(layer, u - ur); return; }
      ps.x11_unit(layer, u - ur);
    });
  }
  FBX_MARK(8);
  if (!P.n_ragged) return;  // (list operators need a ragged input somewhere below them)

  // ---- one-launch mode: the tile's bases come from the tiles before it.  The count went out
  // long ago, so the tiles before this one have had time to count.
  if (MODE == 2) {
    if (wave < P.n_ragged && !row_follows(P, sh, wave) && !lb_place_row(P, sh, tile, wave, early) && lane == 0) s_good = 0u;
    constexpr uint32_t kRows = 4;  // further operators: a wavefront looks back for several at the same time
    for (uint32_t row0 = wave + kWaves; row0 < P.n_ragged; row0 += kRows * kWaves) {
      uint64_t v[kRows];
#pragma unroll
      for (uint32_t k = 0; k < kRows; ++k) {
        const uint32_t row = row0 + k * kWaves;
        v[k] = row < P.n_ragged && !row_follows(P, sh, row) ? lb_window(P, row, tile) : kLbPrefix;
      }
#pragma unroll
      for (uint32_t k = 0; k < kRows; ++k) {
        const uint32_t row = row0 + k * kWaves;
        if (row < P.n_ragged && !row_follows(P, sh, row) && !lb_place_row(P, sh, tile, row, v[k]) && lane == 0) s_good = 0u;
      }
    }
    __syncthreads();
    FBX_MARK(9);
    if (!s_good) return;  // the call fails or falls back: leave the arrays alone
  } else if (MODE == 3 && !ragged_roots_done) {  // (a plan of one layer: the bases taken before phase C are read from here on)
    __syncthreads();
    if (!s_good) return;
  } else if (P.n_mh && !ragged_roots_done) {
    __syncthreads();  // the item index space laid out in phase C is read by every wavefront
  }
  // ---- ragged root operators
  if (!ragged_roots_done) for_units(&s_ctr[3], ragged_root_units(), ragged_root_unit);
  FBX_MARK(10);
  // ---- the list crosses / concats, layer by layer
  for (uint32_t layer = 2, turn = 0; layer <= P.n_layers; ++layer) {
    const uint32_t list = ps.gen_list(layer);
    if (sh.lbeg(list + 1) == sh.lbeg(list)) continue;  // (no such operator in this layer: no barrier either)
    __syncthreads();  // the layer barrier
    uint32_t* ctr = &s_ctr[7u + (turn & 1u)];
    if (tid == 0) s_ctr[7u + ((turn + 1u) & 1u)] = 0;  // the counter of the next layer that has any (idle since the barrier before this one)
    ++turn;
    for_units(ctr, ps.gen_units(layer), [&](uint32_t u) {
      if (!FBX_SKIP(2u)) ps.gen_unit(layer, u);
    });
  }
}

// ------------------------------------------------------------------- kernel
// Copies n bytes (a multiple of 4) from memory into LDS, all lanes taking part.
__device__ __forceinline__ void copy_table(uint8_t* dst, const void* src, uint32_t n) {
  const FBX_GLOBAL uint32_t* s32 = gptr(reinterpret_cast<const uint32_t*>(src));
  uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
  for (uint32_t i = threadIdx.x; i < (n >> 2); i += kTileThreads) d32[i] = s32[i];
}

// Sixteen raw bytes at address ca; what lies outside the caller's buffer reads as zero.
__device__ __forceinline__ u32x4 load_chunk(uintptr_t ca, uintptr_t ok_lo, uintptr_t ok_hi) {
  u32x4 v;
  if (ca >= ok_lo && ca + 16u <= ok_hi) {
    v = *gptr<const u32x4>((uint64_t)ca);
  } else {  // the chunk straddles an end of the buffer: take what exists byte by byte
    uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
    for (uint32_t i = 0; i < 16; ++i) {
      const uintptr_t bi = ca + i;
      uint32_t b = 0;
      if (bi >= ok_lo && bi < ok_hi) b = (uint32_t)*gptr<const uint8_t>((uint64_t)bi) << (8u * (i & 3u));
      const uint32_t q = i >> 2;
      w0 |= q == 0 ? b : 0u; w1 |= q == 1 ? b : 0u; w2 |= q == 2 ? b : 0u; w3 |= q == 3 ? b : 0u;
    }
    v.x = w0; v.y = w1; v.z = w2; v.w = w3;
  }
  return v;
}

// Workgroups are persistent: each copies the plan tables into LDS once and then
// takes tiles off a shared counter until none is left.
template <int MODE>
__device__ __forceinline__ void tile_body(const TileParams& P) {
  constexpr bool WRITE = MODE != 0;
  __shared__ uint32_t s_err, s_len, s_cur, s_nxt;
  __shared__ uint32_t s_bad[2];  // what is wrong with the offsets of the current and of the next tile (CE_ bits)
  Sh sh_ = views(P);
#ifndef FBX_FIXED_MODE
  for (uint32_t i = 0; i <= (uint32_t)TL_LAYER; ++i) sh_.lb[i] = P.list_begin[i];  // (n_lists >= TL_LAYER: always there)
#endif
  const Sh& sh = sh_;
  const uint32_t tid = threadIdx.x;
  const uint32_t T = 1u << P.log2T;
  const FBX_GLOBAL uint64_t* rec_off = gptr(P.rec_off);
  uint32_t* ticket = &P.ctrl->ticket[WRITE ? 1 : 0];  // (MODE 2 needs the order the counter gives: see lb_place_row)
  const uintptr_t ok_lo = reinterpret_cast<uintptr_t>(P.raw), ok_hi = ok_lo + P.raw_len;
  // Tiles are taken off a counter.  A workgroup takes its next tile when it starts on the
  // current one (that early, so that the next tile's offsets and text can be on their way),
  // never more than one ahead: tiles are then started in the order of their numbers, give
  // or take how long single tiles take, which is what the one-launch placement needs.
  if (tid == 0) {
    s_err = P.ctrl->err;  // set by an earlier kernel of this call: nothing may be written
    s_cur = atomicAdd(ticket, 1u);
    s_bad[0] = s_bad[1] = 0;
  }
  {  // the operators' programs in the order of the work lists, their inputs a and b renumbered alike
    static_assert(sizeof(OpProg) == 64 && offsetof(OpProg, a) == 24 && offsetof(OpProg, b) == 28, "OpProg layout");
    const FBX_GLOBAL uint32_t* from = gptr(reinterpret_cast<const uint32_t*>(P.prog));
    const FBX_GLOBAL uint32_t* lists = gptr(P.lists);
    uint32_t* to = reinterpret_cast<uint32_t*>(smem + P.o_prog);
    for (uint32_t i = tid; i < P.n_ops * 16u; i += kTileThreads) {
      const uint32_t w = i & 15u;
      uint32_t v = from[lists[i >> 4] * 16u + w];
      if (w == 6u || w == 7u) {  // a, b
        const uint32_t kind = from[lists[i >> 4] * 16u];
        if ((kind == OP_CROSS || kind == OP_CONCAT) && v < P.n_ops) v = lists[P.n_ops + v];
      }
      to[i] = v;
    }
  }
  copy_table(smem + P.o_lbeg, P.list_begin, (P.n_lists + 1u) * 4u);
  copy_table(smem + P.o_rnr, P.rnr, P.rnr_words * 4u);
  copy_table(smem + P.o_aux, P.aux, P.aux_bytes);
  if (MODE >= 2) copy_table(smem + P.o_cap, P.row_cap, P.n_ragged * 8u);
#ifdef FBX_TILE_PROF
  if (tid < 16) s_prof[tid] = 0;
  if (tid == 0) s_prof_last = clock64();
#endif
  __syncthreads();
  if (s_err) return;
  // Offsets are checked before a tile touches the text: non-decreasing, inside the text, a record shorter than 2 GiB.
  auto offsets_fault = [&](uint64_t a, uint64_t b) -> uint32_t {
    if (a > b || b > P.raw_len) return CE_OFFSETS;
    return b - a >= (1ull << 31) ? CE_TILE : 0u;
  };
  // the first tile's offsets arrive the plain way
  uint32_t par = 0;
  if (s_cur < P.n_tiles) {
    const uint64_t g0 = (uint64_t)s_cur << P.log2T;
    const uint32_t nrec = (uint32_t)min((uint64_t)T, P.n_records - g0);
    if (tid <= nrec) sh.off[tid] = rec_off[g0 + tid];
    if (tid < nrec) {
      const uint32_t bad = offsets_fault(rec_off[g0 + tid], rec_off[g0 + tid + 1]);
      if (bad) atomicOr(&s_bad[0], bad);
    }
  }
  __syncthreads();
  FBX_MARK(0);

  uint32_t malformed = 0;
  bool overflow = false;
  uint32_t tile = s_cur;
  for (;;) {
    if (tile >= P.n_tiles) break;
    uint32_t my_ticket = 0;
    // One-launch mode on a plan of one layer: a tile has little to do between publishing its counts and
    // needing its bases, so it matters that the tiles before it are counted by then.  Tiles whose numbers
    // are taken a whole tile ahead start in an order that has drifted by the time they run (tiles differ
    // in length); there the next tile's number is taken when this tile is done, at the price of fetching
    // its offsets and text with nothing to hide behind (the largest one-layer workload: 5 % faster; a
    // two-layer plan, whose single crosses sit between counts and bases: 7 % slower, so it keeps the early ticket).
    const bool late_ticket = MODE == 2 && P.n_layers == 1u;
    if (!late_ticket && tid == 0) my_ticket = atomicAdd(ticket, 1u);  // the next tile; the answer is picked up a barrier later
    uint64_t* off = sh.off + par * (T + 1u);
    uint64_t* off2 = sh.off + (par ^ 1u) * (T + 1u);
    const uint64_t g0 = (uint64_t)tile << P.log2T;
    const uint32_t nrec = (uint32_t)min((uint64_t)T, P.n_records - g0);
    for (uint32_t row = tid; row < P.n_ragged; row += kTileThreads) {
      sh.run[row] = 0;
      if (MODE == 1) sh.base[row] = gptr(P.tile_base)[(uint64_t)row * P.n_tiles + tile];
    }
    if (tid < 9) s_ctr[tid] = 0;
    if (tid == 9) s_done = 0;
    if (tid == 10) s_good = 1u;
    if (tid == 11) s_absurd = 0u;
    bool nrec_ok = true;
    const uint32_t bad = s_bad[par];  // (found while the tile before this one was worked on)
    if (tid == 0) s_bad[par ^ 1u] = 0;
    if (bad) {
      if (tid == 0) atomicOr(&P.ctrl->err, bad);
      if (MODE != 2) break;  // the call fails: no point in working off the other tiles
      // without a counting launch later tiles wait for this one: tell them, then go on
      lb_abort_tile(P, tile);
      nrec_ok = false;
    }
    FBX_MARK(1);

    // The next tile arrives in steps, one per barrier of this tile, so that no step waits for
    // memory: (0) its number, (1) its record offsets are requested, (2) they are parked in LDS
    // and one byte of every 128-byte line of its text is requested, which brings the text into
    // the L2 cache without holding registers for it.  Only the two outer offsets decide what is
    // touched; the tile itself is checked when its turn comes.
    uint32_t pf_stage = 0, nxt = 0xffffffffu, nrec2 = 0, touch = 0;
    uint64_t off_next = 0, off_next1 = 0, nx_lo = 0, nx_hi = 0;
    auto next_tile_step = [&]() {  // every lane, right after a barrier
      if (pf_stage == 0) {
        if (tid == 0) s_nxt = late_ticket ? atomicAdd(ticket, 1u) : my_ticket;
      } else if (pf_stage == 1) {
        nxt = s_nxt;
        if (nxt < P.n_tiles) {
          const uint64_t g1 = (uint64_t)nxt << P.log2T;
          nrec2 = (uint32_t)min((uint64_t)T, P.n_records - g1);
          if (tid <= nrec2) off_next = rec_off[g1 + tid];
          if (tid < nrec2) off_next1 = rec_off[g1 + tid + 1u];
          nx_lo = rec_off[g1];
          nx_hi = rec_off[g1 + nrec2];
        }
      } else if (pf_stage == 2) {
        if (nxt < P.n_tiles) {
          if (tid <= nrec2) off2[tid] = off_next;
          if (tid < nrec2) {
            const uint32_t fault = offsets_fault(off_next, off_next1);
            if (fault) atomicOr(&s_bad[par ^ 1u], fault);
          }
          if (nx_lo <= nx_hi && nx_hi <= P.raw_len) {
            const uintptr_t first = ok_lo + nx_lo, end = ok_lo + nx_hi;
            const uintptr_t line = (first & ~(uintptr_t)127) + 128u * tid;  // (tiles beyond 64 KiB of text: the first 64 KiB)
            if (line < end) touch = *gptr<const uint8_t>((uint64_t)max(line, first));
          }
        }
      }
      if (pf_stage < 3) ++pf_stage;
    };
    auto next_tile_hook = [&]() {  // (what the phases of a pass call after their barriers)
      if (!late_ticket) next_tile_step();
    };

    uint32_t r0 = nrec_ok ? 0u : nrec;
    if (MODE >= 2 && nrec_ok) {
      // placement needs the whole tile's counts at once: a tile that takes several passes
      // (or holds a record that is read in place) sends the call back to the counting launch
      const uint32_t d0 = (uint32_t)((ok_lo + off[0]) & 15u);
      if (off[nrec] - off[0] + d0 > (uint64_t)P.raw_cap) {
        if (tid == 0) atomicOr(&P.ctrl->err, (uint32_t)(CE_SPEC | CE_PASSES));
        if (MODE == 2) lb_abort_tile(P, tile);
        r0 = nrec;
      }
    }
    while (r0 < nrec) {  // one turn per pass; all conditions are uniform over the workgroup
      const uint64_t o0 = off[r0];
      const uintptr_t addr0 = ok_lo + o0;
      const uint32_t delta = (uint32_t)(addr0 & 15u);
      // the pass takes records r0 .. r1-1: as many as fit the LDS section
      uint32_t lo = r0, hi = nrec;
      if (off[nrec] - o0 + delta <= (uint64_t)P.raw_cap) lo = nrec;  // the usual case: all that is left fits
      while (lo < hi) {
        const uint32_t mid = (lo + hi + 1u) >> 1;
        if (off[mid] - o0 + delta <= (uint64_t)P.raw_cap) lo = mid; else hi = mid - 1u;
      }
      const uint32_t r1 = lo;
      if (r1 > r0) {
        const uint32_t nb = r1 - r0;
        const uint32_t nchunks = (delta + (uint32_t)(off[r1] - o0) + 15u) >> 4;
        const uintptr_t a0 = addr0 - delta;
        if (a0 >= ok_lo && a0 + 16ull * nchunks <= ok_hi) {  // whole chunks (all but the ends of the caller's buffer)
          const FBX_GLOBAL u32x4* from = gptr<const u32x4>((uint64_t)a0);
          for (uint32_t c = tid; c < nchunks; c += kTileThreads)
            *reinterpret_cast<u32x4*>(sh.raw + kRawPad + 16u * c) = from[c];
        } else {
          for (uint32_t c = tid; c < nchunks; c += kTileThreads)
            *reinterpret_cast<u32x4*>(sh.raw + kRawPad + 16u * c) = load_chunk(a0 + 16u * c, ok_lo, ok_hi);
        }
        if (tid < nb) {
          sh.rs[tid] = kRawPad + delta + (uint32_t)(off[r0 + tid] - o0);
          sh.re[tid] = kRawPad + delta + (uint32_t)(off[r0 + tid + 1] - o0);
        }
        __syncthreads();
        FBX_MARK(2);
        if (!FBX_SKIP(8u)) tokenize(P, sh, nb);
        if (FBX_SKIP(0x100u)) {  // (tuning builds: once more, to weigh it)
          __syncthreads();
          tokenize(P, sh, nb);
        }
        __syncthreads();
        FBX_MARK(3);
        LdsSrc src{sh.raw, sh.rows, P.row_stride};
        run_pass<MODE>(P, sh, src, nb, g0 + r0, tile, malformed, overflow, next_tile_hook);
        r0 = r1;
      } else {
        // record r0 alone exceeds the section: it is read in place
        const uint64_t len64 = off[r0 + 1] - o0;
        if (tid == 0) {
          uint32_t len = (uint32_t)len64;
          if (len && gptr(P.raw)[o0 + len - 1u] == '\n') --len;
          s_len = len;
        }
        __syncthreads();
        GlobalSrc src{gptr(P.raw) + o0, s_len};
        run_pass<MODE>(P, sh, src, 1u, g0 + r0, tile, malformed, overflow, next_tile_hook);
        r0 += 1u;
      }
      __syncthreads();  // the sections are reused by the next pass
      if (tid < 9) s_ctr[tid] = 0;
      if (tid == 9) s_done = 0;
      if (tid == 10) s_good = 1u;
      if (tid == 11) s_absurd = 0u;
      FBX_MARK(11);
    }
    if (!WRITE) {
      for (uint32_t row = tid; row < P.n_ragged; row += kTileThreads)
        gptr(P.tile_cnt)[(uint64_t)row * P.n_tiles + tile] = sh.run[row];
    }
    if (pf_stage < 3) {  // (a tile with few barriers: the remaining steps each get their own)
      do {
        __syncthreads();
        next_tile_step();
      } while (pf_stage < 3);
      __syncthreads();  // the parked offsets are read by other lanes
    }
    asm volatile("" ::"v"(touch));  // the touched byte itself is of no use
    par ^= 1u;
    tile = nxt;  // every lane has read the ticket by now
    FBX_MARK(12);
  }

#ifdef FBX_TILE_PROF
  __syncthreads();
  if (tid < 16 && P.prof) atomicAdd(reinterpret_cast<unsigned long long*>(P.prof) + tid + (WRITE ? 16 : 0), s_prof[tid]);
#endif
  if (!WRITE) {
    if (overflow) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
  } else {
    if (MODE >= 2 && overflow) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
    for (int d = 32; d >= 1; d >>= 1) malformed += __shfl_xor(malformed, d, 64);
    if (lane_id() == 0 && malformed)
      atomicAdd(reinterpret_cast<unsigned long long*>(&P.ctrl->n_malformed), (unsigned long long)malformed);
  }
}

#ifndef FBX_FIXED_MODE
// ---- one ragged root operator with in-kernel allocation, results behind per-record pointers
// Section 5 as the paper uses it (Figure 5): a thread works out how much memory its result needs,
// the workgroup allocates with Algorithm 1 (one atomic add per workgroup, arena_alloc_wg), the
// thread writes its result into its region and leaves the region's offset in the table of thread
// offsets.  One record per thread, read in place; no counting launch, no scan.  Regions of one
// workgroup lie end to end in record order; workgroups land in the order in which they arrive.
__global__ __launch_bounds__(kBlock) void k_unordered(UnorderedParams U) {
  __shared__ uint64_t s_part[kBlock / 64 + 2];
  const uint64_t r = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const OpProg& d = U.op;
  bool ok = r < U.n_records;
  uint32_t cnt = 0, s = 0, e = 0, err = 0;
  GlobalSrc src{gptr(U.raw), 0u};
  if (ok) {
    const uint64_t a = U.rec_off[r], b = U.rec_off[r + 1];
    if (a > b || b > U.raw_len) { err = CE_OFFSETS; ok = false; }
    else if (b - a >= (1ull << 31)) { err = CE_TILE; ok = false; }
    else {
      uint32_t len = (uint32_t)(b - a);
      if (len && U.raw[b - 1] == '\n') --len;
      src = GlobalSrc{gptr(U.raw) + a, len};
      src.span(0, d.field, s, e);
      if (d.kind == OP_NGRAM) cnt = e - s >= d.aux_len ? e - s - d.aux_len + 1u : 0u;
      else cnt = (d.kind == OP_FILTER && (d.flags & F_NEVER)) ? 0u : ragged_root_count(src, d, U.aux, s, e);
      if (cnt > kMaxCount) { err = CE_OVERFLOW; ok = false; cnt = 0; }
    }
  }
  const uint64_t off = arena_alloc_wg(&U.state[0], 8ull * cnt, s_part);  // (every thread of the workgroup)
  uint32_t malformed = 0;
  if (r < U.n_records) {
    U.thread_off[r] = ok ? off : 0ull;
    U.lengths[r] = cnt;
  }
  if (ok && cnt) {
    if (off + 8ull * cnt > U.pool_bytes) {
      err = CE_NOMEM;  // the pool is exhausted: nothing is written beyond it, the head says what would have sufficed
    } else {
      G64 dst = gptr(reinterpret_cast<uint64_t*>(U.pool + off));
      if (d.kind == OP_NGRAM) {
        for (uint32_t q = 0; q < cnt; ++q) dst[q] = hash_span(src, s + q, s + q + d.aux_len, d.key);
      } else {
        ragged_root_emit(src, d, U.aux, s, e, dst, malformed);
      }
    }
  }
  if (err) atomicOr(reinterpret_cast<unsigned long long*>(&U.state[1]), (unsigned long long)err);
  uint64_t total = cnt;
  for (int sh = 32; sh >= 1; sh >>= 1) {
    total += __shfl_xor(total, sh, 64);
    malformed += __shfl_xor(malformed, sh, 64);
  }
  if ((threadIdx.x & 63u) == 0) {
    if (total) atomicAdd(reinterpret_cast<unsigned long long*>(&U.state[2]), (unsigned long long)total);
    if (malformed) atomicAdd(reinterpret_cast<unsigned long long*>(&U.state[3]), (unsigned long long)malformed);
  }
}

// The kernel for any plan: everything it needs to know arrives in P.
template <int MODE>
__global__ __launch_bounds__(kTileThreads, 4) void k_tile(TileParams P) {
  tile_body<MODE>(P);
}
#endif

}  // namespace

#ifdef FBX_FIXED_MODE
// The kernel for one plan and one shape of tile, compiled when the plan first meets that shape
// (the meta-kernel of Section 4, with this file as its template): FBX_FIXED_ASSIGN sets the
// fields of P that the plan and the tile size fix (counts, LDS offsets, tile size) to literal
// values, so that loops over layers and lists unroll or vanish, the LDS sections have constant
// addresses and far fewer values compete for scalar registers.  The launch checks that the
// fields it passes are the ones compiled in.
// (its name, FBX_FIXED_NAME, ends in the mode, so that a trace tells the three kernels apart)
#ifndef FBX_FIXED_WAVES
#define FBX_FIXED_WAVES 4
#endif
// (the kernels that write are compiled for size: 1-3 % faster on the largest workload, none slower; the
// counting kernel is 3 % slower that way and stays as it is)
#if FBX_FIXED_MODE != 0
#define FBX_SIZE_ATTR __attribute__((minsize))
#else
#define FBX_SIZE_ATTR
#endif
extern "C" __global__ __launch_bounds__(kTileThreads, FBX_FIXED_WAVES) FBX_SIZE_ATTR void FBX_FIXED_NAME(TileParams Pin) {
  TileParams P = Pin;
  FBX_FIXED_ASSIGN
  tile_body<FBX_FIXED_MODE>(P);
}
#endif

#if !defined(__HIPCC_RTC__) && !defined(FBX_FIXED_MODE)
// ----------------------------------------------------------- launch wrappers
uint32_t tile_max_lds() {
  static uint32_t cached = 0;
  if (!cached) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
      cached = (uint32_t)v;
    else
      cached = 160u * 1024u;  // (no device to ask, as when a plan's kernel source is only written out: gfx950's)
  }
  return cached;
}

hipError_t launch_tile(const TileParams& P, int mode, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  const void* fn = mode == 0   ? reinterpret_cast<const void*>(&k_tile<0>)
                   : mode == 1 ? reinterpret_cast<const void*>(&k_tile<1>)
                   : mode == 2 ? reinterpret_cast<const void*>(&k_tile<2>)
                               : reinterpret_cast<const void*>(&k_tile<3>);
  if (P.lds_bytes > 48u * 1024u) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)P.lds_bytes);
    if (e != hipSuccess) return e;
  }
  // as many workgroups as can run at the same time (the one-launch mode relies on it)
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kTileThreads, P.lds_bytes) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    per_cu = 1;
  }
  uint32_t capacity = tile_cu_count() * (uint32_t)per_cu;
  if (P.grid && P.grid < capacity) capacity = P.grid;
  TileParams Q = P;
  const uint32_t grid = std::min(P.n_tiles, capacity);
  if (mode == 0) hipLaunchKernelGGL(k_tile<0>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, Q);
  else if (mode == 1) hipLaunchKernelGGL(k_tile<1>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, Q);
  else if (mode == 2) hipLaunchKernelGGL(k_tile<2>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, Q);
  else hipLaunchKernelGGL(k_tile<3>, dim3(grid), dim3(kTileThreads), P.lds_bytes, st, Q);
  return hipGetLastError();
}

hipError_t launch_unordered(const UnorderedParams& U, hipStream_t st) {
  if (U.n_records == 0) return hipSuccess;
  const uint64_t blocks = (U.n_records + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(k_unordered, dim3((uint32_t)blocks), dim3(kBlock), 0, st, U);
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
#endif  // __HIPCC_RTC__

}  // namespace fbx
