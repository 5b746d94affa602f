// The walk kernels of libfbx for gfx950 (MI355X): counting pass and writing pass.
//
// Work decomposition.  Records are independent (every operator computes on one
// row of the table; Section 3, "Extract features"), so one wavefront owns a tile
// of 64 consecutive records, one record per lane, and walks the fields of its
// records in lock step: field 0 of all 64 records, then field 1, and so on.
// Which operators read field k is the same for every record, so all control
// flow that depends on the plan is wave-uniform and runs on the scalar unit; a
// lane only diverges from its neighbours by the length of its own field.
//
//  * Raw bytes are read in place: a lane loads a 16-byte window at its current
//    position (4-byte aligned, funnel-shifted into place) and takes its bytes
//    out of registers.  The 64 windows of a wavefront lie in 64 different
//    records; they are served by L2, and every raw byte comes from HBM once.
//  * Splitting at the delimiter (Section 5, first paragraph) needs no array
//    here: the end of a field is found by the same loop that hashes it.
//  * A fixed-arity slot is written by 64 lanes to 64 consecutive u64: one
//    512-byte store per wavefront and operator.
//  * A ragged slot needs the tile's base inside the slot (from the counting
//    pass and the scan over tiles) plus a prefix sum over the 64 lanes.
//  * Later layers run in the same lane on the signs that lane wrote itself, so
//    executing all layers in one launch needs no synchronisation between
//    wavefronts at all; the per-layer launch of the paper (Section 4) is the
//    same kernel restricted to one layer.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "fbx_device.h"

namespace fbx {

constexpr uint32_t kNoRow = 0xffffffffu;
constexpr uint64_t kPrime = 0x100000001b3ull;
constexpr uint32_t kWin = 12;  // bytes of a window that are always valid after alignment

// ------------------------------------------------------------ small helpers
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  const uint32_t lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d, 64);
    if (lane >= (uint32_t)d) v += t;
  }
  return v;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// Load of a table record that every lane of the wavefront reads alike and that
// no kernel writes while this one runs (plan tables, and per-call tables written
// by earlier kernels of the same stream).  Going through the constant address
// space lets the compiler use scalar loads, which do not wait on the vector
// memory counter and land in SGPRs.
#define FBX_CONST __attribute__((address_space(4)))
#define FBX_GLOBAL __attribute__((address_space(1)))
// An address kept as an integer, turned back into a pointer the compiler knows to be global memory.
template <class T>
__device__ __forceinline__ FBX_GLOBAL T* gptr(uint64_t addr) { return reinterpret_cast<FBX_GLOBAL T*>(addr); }
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
using G64 = FBX_GLOBAL uint64_t*;         // signs and offsets being written
using CG64 = const FBX_GLOBAL uint64_t*;  // signs and offsets being read
template <class T>
__device__ __forceinline__ T cload(const T* p) {
  static_assert(sizeof(T) % 4 == 0, "dword multiples only");
  constexpr int N = sizeof(T) / 4;
  const FBX_CONST uint32_t* q = reinterpret_cast<const FBX_CONST uint32_t*>(reinterpret_cast<uintptr_t>(p));
  union { T t; uint32_t w[N]; } u;
#pragma unroll
  for (int i = 0; i < N; ++i) u.w[i] = q[i];
  return u.t;
}

// ------------------------------------------------------------ byte windows
// Per-wavefront view of the raw buffer.  Positions are 32-bit offsets from the
// first byte of the tile (a tile spans less than 2 GiB; checked beforehand).
//
// A lane walks its record front to back a few bytes at a time, and the 64
// records of a wavefront lie far apart, so fetching every 16-byte window from
// memory would pull the same 64-byte sector out of HBM once per window.  Each
// lane therefore keeps the two sectors it is working in inside LDS (a two-entry
// direct-mapped cache, sector s in slot s & 1): a sector is fetched from memory
// once, with four adjacent 16-byte loads, and windows are then cut out of LDS.
// Dword d of a lane's 128 ring bytes sits at ring[d * 64 + lane], so all lanes
// hit different banks whatever their positions; the first three dwords of slot
// 0 are mirrored behind slot 1 so that a window never wraps.
constexpr uint32_t kRingDwords = 35;                 // 2 sectors of 16 dwords + 3 mirrored
constexpr uint32_t kRingWave = kRingDwords * 64u;    // dwords of LDS per wavefront

extern __shared__ __align__(16) uint32_t smem32[];

struct Ctx {
  const FBX_GLOBAL uint8_t* base64;  // 64-byte aligned address at or just before tile byte 0   (uniform)
  uint32_t delta;         // tile byte 0 is base64[delta], delta in 0..63            (uniform)
  uint32_t lo_valid;      // base64[o] lies inside the raw buffer iff lo_valid <= o < hi_valid
  uint32_t hi_valid;
  uint32_t ring;          // index in smem32 of dword 0 of this lane's ring          (per lane)
  uint32_t tag0, tag1;    // sector held in slot 0 / slot 1, 0xffffffff = none       (per lane)
};

struct Win { uint32_t a, b, c; };  // 12 bytes starting at the requested position

// Fetch 64-byte sector s of this lane's stream into its ring slot.
__device__ __forceinline__ void ring_fill(Ctx& c, uint32_t s) {
  const uint32_t so = s << 6;
  uint32_t v[16];
  if (so >= c.lo_valid && so + 64u <= c.hi_valid) {
    const FBX_GLOBAL u32x4* src = reinterpret_cast<const FBX_GLOBAL u32x4*>(c.base64 + so);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 q = src[i];
      v[4 * i] = q.x; v[4 * i + 1] = q.y; v[4 * i + 2] = q.z; v[4 * i + 3] = q.w;
    }
  } else {
    // sector straddles an end of the buffer: fetch what exists byte by byte
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = 0;
    for (uint32_t i = 0; i < 64; ++i) {
      const uint32_t oi = so + i;
      if (oi >= c.lo_valid && oi < c.hi_valid) {
        const uint32_t byte = (uint32_t)c.base64[oi] << (8u * (i & 3u));
#pragma unroll
        for (int k = 0; k < 16; ++k) if ((i >> 2) == (uint32_t)k) v[k] |= byte;
      }
    }
  }
  const uint32_t slot = s & 1u;
  const uint32_t dst = c.ring + slot * 16u * 64u;
#pragma unroll
  for (int i = 0; i < 16; ++i) smem32[dst + i * 64] = v[i];
  if (slot == 0) {
    smem32[c.ring + 32 * 64] = v[0];
    smem32[c.ring + 33 * 64] = v[1];
    smem32[c.ring + 34 * 64] = v[2];
    c.tag0 = s;
  } else {
    c.tag1 = s;
  }
}

__device__ __forceinline__ Win load_win(Ctx& c, uint32_t p) {
  const uint32_t o = p + c.delta, qa = o & ~3u, sh = (o & 3u) * 8u;
  const uint32_t s0 = qa >> 6, s1 = (qa + 15u) >> 6;
  if (((s0 & 1u) ? c.tag1 : c.tag0) != s0) ring_fill(c, s0);
  if (((s1 & 1u) ? c.tag1 : c.tag0) != s1) ring_fill(c, s1);
  const uint32_t idx = c.ring + ((qa >> 2) & 31u) * 64u;
  const uint32_t w0 = smem32[idx], w1 = smem32[idx + 64], w2 = smem32[idx + 128], w3 = smem32[idx + 192];
  Win r;
  r.a = __builtin_amdgcn_alignbit(w1, w0, sh);
  r.b = __builtin_amdgcn_alignbit(w2, w1, sh);
  r.c = __builtin_amdgcn_alignbit(w3, w2, sh);
  return r;
}

// The same window straight from memory, for accesses that do not follow the
// lane's own record (lanes reading neighbouring bytes of one record coalesce).
__device__ __forceinline__ Win load_win_direct(const Ctx& c, uint32_t p) {
  const uint32_t o = p + c.delta, qa = o & ~3u, sh = (o & 3u) * 8u;
  uint32_t w0, w1, w2, w3;
  if (qa >= c.lo_valid && qa + 16u <= c.hi_valid) {
    const FBX_GLOBAL uint32_t* src = reinterpret_cast<const FBX_GLOBAL uint32_t*>(c.base64 + qa);
    w0 = src[0]; w1 = src[1]; w2 = src[2]; w3 = src[3];
  } else {
    uint32_t w[4] = {0, 0, 0, 0};
    for (uint32_t i = 0; i < 16; ++i) {
      const uint32_t oi = qa + i;
      if (oi >= c.lo_valid && oi < c.hi_valid) w[i >> 2] |= (uint32_t)c.base64[oi] << (8u * (i & 3u));
    }
    w0 = w[0]; w1 = w[1]; w2 = w[2]; w3 = w[3];
  }
  Win r;
  r.a = __builtin_amdgcn_alignbit(w1, w0, sh);
  r.b = __builtin_amdgcn_alignbit(w2, w1, sh);
  r.c = __builtin_amdgcn_alignbit(w3, w2, sh);
  return r;
}

__device__ __forceinline__ uint32_t load_byte(const Ctx& c, uint32_t p) { return c.base64[p + c.delta]; }

template <int J>
__device__ __forceinline__ uint32_t win_byte(const Win& w) {
  const uint32_t d = J < 4 ? w.a : (J < 8 ? w.b : w.c);
  return (d >> (8 * (J & 3))) & 0xffu;
}

// 0x80 in (at least) the lowest zero byte of x; bytes above a zero byte may be flagged too.
__device__ __forceinline__ uint32_t zero_low(uint32_t x) { return (x - 0x01010101u) & ~x & 0x80808080u; }
// 0x80 in exactly the zero bytes of x.
__device__ __forceinline__ uint32_t zero_exact(uint32_t x) {
  return ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);
}

// Index of the first tab among the first n (<= 12) bytes of the window, or n.
__device__ __forceinline__ uint32_t first_tab(const Win& w, uint32_t n) {
  const uint32_t t0 = zero_low(w.a ^ 0x09090909u), t1 = zero_low(w.b ^ 0x09090909u), t2 = zero_low(w.c ^ 0x09090909u);
  uint32_t idx = 12;
  if (t2) idx = 8 + ((__ffs(t2) - 1) >> 3);
  if (t1) idx = 4 + ((__ffs(t1) - 1) >> 3);
  if (t0) idx = (__ffs(t0) - 1) >> 3;
  return idx < n ? idx : n;
}

// Number of commas among the first m (<= 12) bytes of the window.
__device__ __forceinline__ uint32_t count_commas(const Win& w, uint32_t m) {
  const uint32_t f[3] = {zero_exact(w.a ^ 0x2c2c2c2cu), zero_exact(w.b ^ 0x2c2c2c2cu), zero_exact(w.c ^ 0x2c2c2c2cu)};
  uint32_t c = 0;
#pragma unroll
  for (int d = 0; d < 3; ++d) {
    const uint32_t v = m > 4u * d ? (m - 4u * d < 4u ? m - 4u * d : 4u) : 0u;  // valid bytes of this dword
    const uint32_t mask = v >= 4u ? 0xffffffffu : ((1u << (8u * v)) - 1u);
    c += __popc(f[d] & mask);
  }
  return c;
}

// End of the field that starts at pos: position of its tab, or the end of the
// record.  With COMMAS the commas of the field are counted on the way.
template <bool COMMAS>
__device__ __forceinline__ uint32_t find_end(Ctx& c, uint32_t pos, uint32_t end, uint32_t& commas) {
  uint32_t p = pos;
  commas = 0;
  while (p < end) {
    const uint32_t n = end - p < kWin ? end - p : kWin;
    const Win w = load_win(c, p);
    const uint32_t i = first_tab(w, n);
    if (COMMAS) commas += count_commas(w, i);
    p += i;
    if (i < n) break;
  }
  return p;
}

// Calls f(byte) for every byte of [s, e), in order.
// Calls f(byte) for the first n (<= 12) bytes of a window, in order.  The steps
// nest (step J+1 sits inside the test of step J), so a lane that is done leaves
// the execution mask once and the wavefront skips ahead when every lane is done.
template <class F>
__device__ __forceinline__ void for_win_bytes(const Win& w, uint32_t n, F&& f) {
#define FBX_OPEN(J) if (n > (uint32_t)J) { f(win_byte<J>(w));
  FBX_OPEN(0) FBX_OPEN(1) FBX_OPEN(2) FBX_OPEN(3) FBX_OPEN(4) FBX_OPEN(5)
  FBX_OPEN(6) FBX_OPEN(7) FBX_OPEN(8) FBX_OPEN(9) FBX_OPEN(10) FBX_OPEN(11)
  }}}}}}}}}}}}
#undef FBX_OPEN
}

// Calls f(byte) for every byte of [s, e), in order.
template <class F>
__device__ __forceinline__ void for_each_byte(Ctx& c, uint32_t s, uint32_t e, F&& f) {
  for (uint32_t p = s; p < e; p += kWin) {
    const uint32_t n = e - p < kWin ? e - p : kWin;
    const Win w = load_win(c, p);
    for_win_bytes(w, n, f);
  }
}

// Single-valued hash of the field at pos, fused with the search for its tab:
// the bytes of a window up to its first tab are folded into h, window by window.
// Returns the position of the field's end (its tab, or the end of the record).
__device__ __forceinline__ uint32_t hash_to_tab(Ctx& c, uint32_t pos, uint32_t end, uint64_t& h) {
  uint32_t p = pos;
  while (p < end) {
    const uint32_t n = end - p < kWin ? end - p : kWin;
    const Win w = load_win(c, p);
    const uint32_t i = first_tab(w, n);
    uint64_t hh = h;
    for_win_bytes(w, i, [&](uint32_t b) { hh = (hh ^ b) * kPrime; });
    h = hh;
    p += i;
    if (i < n) break;
  }
  return p;
}

// ------------------------------------------------------------ token operators
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

template <class D>
__device__ __forceinline__ uint64_t bucket_sign(const D& d, const uint8_t* aux, NumState& ns, uint32_t& malformed) {
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

// Number of signs a ragged root operator (not n-gram) produces on [s, e); commas = #',' in the span.
template <class D>
__device__ __forceinline__ uint32_t ragged_root_count(Ctx& c, const D& d, const uint8_t* aux, uint32_t s,
                                                      uint32_t e, uint32_t commas) {
  if (d.kind != OP_FILTER) return commas + 1;  // multi-valued hash / bucket
  const uint8_t* pre = aux + d.aux_off;
  const uint32_t plen = d.aux_len;
  const bool multi = d.flags & F_MULTI;
  uint32_t cnt = 0, k = 0;
  bool match = true;
  for_each_byte(c, s, e, [&](uint32_t b) {
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

// Writes the signs of a root operator (not n-gram) on [s, e) to dst[0 .. count).
template <class D>
__device__ __forceinline__ void root_emit(Ctx& c, const D& d, const uint8_t* aux, uint32_t s, uint32_t e,
                                          G64 dst, uint32_t& malformed) {
  const bool multi = d.flags & F_MULTI;
  if (d.kind == OP_HASH) {
    uint64_t h = d.key;
    for_each_byte(c, s, e, [&](uint32_t b) {
      if (multi && b == ',') { *dst++ = h; h = d.key; }
      else h = (h ^ b) * kPrime;
    });
    *dst = h;
  } else if (d.kind == OP_FILTER) {
    const uint8_t* pre = aux + d.aux_off;
    const uint32_t plen = d.aux_len;
    uint64_t h = d.key;
    uint32_t k = 0;
    bool match = true;
    for_each_byte(c, s, e, [&](uint32_t b) {
      if (multi && b == ',') {
        if (match && k >= plen) *dst++ = h;
        h = d.key; k = 0; match = true;
      } else {
        if (k < plen && b != pre[k]) match = false;
        h = (h ^ b) * kPrime;
        ++k;
      }
    });
    if (match && k >= plen) *dst = h;
  } else {  // OP_BUCKET
    NumState ns;
    for_each_byte(c, s, e, [&](uint32_t b) {
      if (multi && b == ',') {
        *dst++ = bucket_sign(d, aux, ns, malformed);
        ns = NumState();
      } else ns.step(b);
    });
    *dst = bucket_sign(d, aux, ns, malformed);
  }
}

// ------------------------------------------------------------ tile set-up
struct Tile {
  Ctx ctx;
  uint32_t tile;
  uint64_t g;      // this lane's record
  bool live;       // false in the lanes past the last record
  uint32_t pos, end;
};

// Which tile this wavefront owns.  Consecutive workgroup ids are dealt
// round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so that
// neighbouring tiles, whose outputs share cache lines, share an L2.
__device__ __forceinline__ bool tile_of_wave(uint32_t n_tiles, uint32_t waves_per_block, uint32_t& tile) {
  const uint32_t chunk = gridDim.x >> 3;
  const uint32_t blk = (blockIdx.x & 7u) * chunk + (blockIdx.x >> 3);
  tile = blk * waves_per_block + (threadIdx.x >> 6);
  return tile < n_tiles;
}

__device__ __forceinline__ void open_tile(const WalkParams& P, Tile& t, bool need_raw, uint32_t ring_base) {
  const uint64_t g0 = (uint64_t)t.tile << kTileLog2;
  t.g = g0 + lane_id();
  t.live = t.g < P.n_records;
  t.pos = t.end = 0;
  if (!need_raw) return;
  uint64_t a = 0, b = 0;
  if (t.live) { a = P.rec_off[t.g]; b = P.rec_off[t.g + 1]; }
  const uint64_t tile_lo = uniform64(a);  // lane 0 is always live
  const uintptr_t t0 = reinterpret_cast<uintptr_t>(P.raw) + tile_lo;
  const uintptr_t base64 = t0 & ~uintptr_t(63);
  const uintptr_t raw0 = reinterpret_cast<uintptr_t>(P.raw);
  t.ctx.base64 = gptr<const uint8_t>(base64);
  t.ctx.delta = (uint32_t)(t0 & 63u);
  t.ctx.lo_valid = raw0 > base64 ? (uint32_t)(raw0 - base64) : 0u;
  const uint64_t hi = raw0 + P.raw_len - base64;
  t.ctx.hi_valid = hi > 0xffffffffull ? 0xffffffffu : (uint32_t)hi;
  t.ctx.ring = ring_base + lane_id();
  t.ctx.tag0 = t.ctx.tag1 = 0xffffffffu;
  if (t.live) {
    t.pos = (uint32_t)(a - tile_lo);
    t.end = (uint32_t)(b - tile_lo);
    // one trailing newline is not part of the record
    if (t.end > t.pos && load_byte(t.ctx, t.end - 1) == '\n') --t.end;
  }
}

// Base of this tile inside a ragged operator's value array plus the lane's
// exclusive prefix: where the lane's signs start.  Also writes the lane's two
// offsets entries (each lane writes its own end too, so that a lane can later
// read back both of its entries without relying on a neighbour).
__device__ __forceinline__ uint64_t place_ragged(const WalkParams& P, const Tile& t, const OpProg& d, uint32_t cnt) {
  const uint32_t incl = wave_incl_scan(cnt);
  const uint64_t start = cload(&P.tile_base[(uint64_t)d.rag_row * P.n_tiles + t.tile]) + (incl - cnt);
  if (t.live) {
    G64 off = gptr<uint64_t>(d.offsets);
    off[t.g] = start;
    off[t.g + 1] = start + cnt;
  }
  return start;
}

// This lane's list of an earlier operator.
__device__ __forceinline__ void input_list(const OpProg& d, uint64_t g, CG64& ptr, uint32_t& n) {
  CG64 vals = gptr<const uint64_t>(d.values);
  if (d.arity) {
    n = d.arity;
    ptr = vals + g * d.arity;
  } else {
    CG64 off = gptr<const uint64_t>(d.offsets);
    const uint64_t o0 = off[g], o1 = off[g + 1];
    n = (uint32_t)(o1 - o0);
    ptr = vals + o0;
  }
}

// ------------------------------------------------------------ counting pass
// Per tile and ragged operator: how many signs the tile's 64 records produce.
// Dynamic LDS: the byte rings of the wavefronts, then one row of 64 u32 per ragged operator and wavefront.
__global__ __launch_bounds__(kBlock) void k_count(WalkParams P) {
  if (P.ctrl->err) return;  // an earlier kernel of this call found a problem
  Tile t;
  if (!tile_of_wave(P.n_tiles, P.waves_per_block, t.tile)) return;
  const uint32_t wave = threadIdx.x >> 6;
  open_tile(P, t, true, wave * kRingWave);
  const uint32_t lane = lane_id();
  // after the rings: one row of 64 counts per ragged operator, [row][lane], per wavefront
  uint32_t* cnt = smem32 + P.waves_per_block * kRingWave + (size_t)wave * P.n_ragged * 64u;
  for (uint32_t k = 0; k < P.count_fields; ++k) {
    const FieldDesc fd = cload(&P.fields[k]);
    uint32_t commas, e;
    if (fd.need & 1u) e = find_end<true>(t.ctx, t.pos, t.end, commas);
    else e = find_end<false>(t.ctx, t.pos, t.end, commas);
    for (uint32_t q = 0; q < fd.op_count; ++q) {
      const OpDesc d = cload(&P.ops[cload(&P.field_ops[fd.op_begin + q])]);
      if (d.rag_row == kNoRow) continue;
      uint32_t c;
      if (d.kind == OP_NGRAM) {
        const uint32_t L = e > t.pos ? e - t.pos : 0u;
        c = L >= d.aux_len ? L - d.aux_len + 1 : 0u;
      } else {
        c = ragged_root_count(t.ctx, d, P.aux, t.pos, e, commas);
      }
      cnt[d.rag_row * 64u + lane] = t.live ? c : 0u;
    }
    t.pos = e + 1;
  }
  // counts of the later layers follow from the inputs' counts, record by record
  bool overflow = false;
  for (uint32_t k = 0; k < P.n_nonroot; ++k) {
    const OpDesc d = cload(&P.ops[cload(&P.nonroot[k])]);
    if (d.rag_row == kNoRow) continue;
    const OpDesc da = cload(&P.ops[d.a]);
    const OpDesc db = cload(&P.ops[d.b]);
    const uint64_t ca = da.arity ? da.arity : cnt[da.rag_row * 64u + lane];
    const uint64_t cb = db.arity ? db.arity : cnt[db.rag_row * 64u + lane];
    const uint64_t c = d.kind == OP_CROSS ? ca * cb : ca + cb;
    if (c > 0x3ffffffull) overflow = true;  // keeps a tile's total below 2^32
    cnt[d.rag_row * 64u + lane] = t.live ? (uint32_t)c : 0u;
  }
  for (uint32_t row = 0; row < P.n_ragged; ++row) {
    const uint32_t c = cnt[row * 64u + lane];
    if (c > 0x3ffffffu) overflow = true;
    const uint64_t sum = wave_sum64(c);
    if (lane == 0) P.tile_cnt[(uint64_t)row * P.n_tiles + t.tile] = (uint32_t)sum;
  }
  if (overflow) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
}

// ------------------------------------------------------------- writing pass
__device__ __forceinline__ void walk_roots(const WalkParams& P, Tile& t, uint32_t& malformed) {
  const uint32_t lane = lane_id();
  FieldProg next = cload(&P.prog_fields[0]);
  for (uint32_t k = 0; k < P.n_fields; ++k) {
    const FieldProg fd = next;
    if (k + 1 < P.n_fields) next = cload(&P.prog_fields[k + 1]);  // in flight while this field is worked on
    if (fd.cls == FC_HASH1) {
      uint64_t h = fd.key;
      const uint32_t e = hash_to_tab(t.ctx, t.pos, t.end, h);
      if (t.live) gptr<uint64_t>(fd.dst)[t.g] = h;
      t.pos = e + 1;
      continue;
    }
    uint32_t commas, e;
    if (fd.need & 1u) e = find_end<true>(t.ctx, t.pos, t.end, commas);
    else e = find_end<false>(t.ctx, t.pos, t.end, commas);
    for (uint32_t q = 0; q < fd.op_count; ++q) {
      const OpProg d = cload(&P.prog_ops[cload(&P.field_ops[fd.op_begin + q])]);
      G64 vals = gptr<uint64_t>(d.values);
      if (d.kind == OP_NGRAM) {
        // lanes over the grams of one record at a time: balanced and coalesced
        const uint32_t L = e > t.pos ? e - t.pos : 0u;
        const uint32_t n = d.aux_len;
        const uint32_t ng = (t.live && L >= n) ? L - n + 1 : 0u;
        const uint64_t start = place_ragged(P, t, d, ng);
        for (int r = 0; r < kTile; ++r) {
          const uint32_t ng_r = __shfl(ng, r, 64);
          if (ng_r == 0) continue;
          const uint32_t s_r = __shfl(t.pos, r, 64);
          const uint64_t start_r = __shfl(start, r, 64);
          for (uint32_t g = lane; g < ng_r; g += 64) {
            const Win w = load_win_direct(t.ctx, s_r + g);
            uint64_t h = d.key;
#define FBX_STEP(J) if ((uint32_t)J < n) h = (h ^ win_byte<J>(w)) * kPrime;
            FBX_STEP(0) FBX_STEP(1) FBX_STEP(2) FBX_STEP(3) FBX_STEP(4) FBX_STEP(5) FBX_STEP(6) FBX_STEP(7)
#undef FBX_STEP
            vals[start_r + g] = h;
          }
        }
        continue;
      }
      G64 dst;
      if (d.arity) {
        dst = vals + t.g;  // single-valued hash or bucket: arity 1
      } else {
        const uint32_t c = t.live ? ragged_root_count(t.ctx, d, P.aux, t.pos, e, commas) : 0u;
        dst = vals + place_ragged(P, t, d, c);
      }
      if (t.live) root_emit(t.ctx, d, P.aux, t.pos, e, dst, malformed);  // a filter that keeps nothing writes nothing
    }
    t.pos = e + 1;
  }
}

__device__ __forceinline__ void run_layer(const WalkParams& P, const Tile& t, uint32_t layer) {
  const uint32_t l0 = cload(&P.layer_begin[layer - 1]), l1 = cload(&P.layer_begin[layer]);
  for (uint32_t q = l0; q < l1; ++q) {
    const OpProg d = cload(&P.prog_ops[cload(&P.layer_ops[q])]);
    const OpProg da = cload(&P.prog_ops[d.a]);
    const OpProg db = cload(&P.prog_ops[d.b]);
    G64 vals = gptr<uint64_t>(d.values);
    if (d.kind == OP_CROSS && da.arity == 1 && db.arity == 1) {
      // the common case: two single-valued inputs, one sign out, all three accesses coalesced
      if (t.live) {
        const uint64_t a = gptr<const uint64_t>(da.values)[t.g];
        const uint64_t b = gptr<const uint64_t>(db.values)[t.g];
        vals[t.g] = mix64(mix64(a + d.key) + b);
      }
      continue;
    }
    CG64 pa = nullptr; CG64 pb = nullptr;
    uint32_t na = 0, nb = 0;
    if (t.live) {
      input_list(da, t.g, pa, na);
      input_list(db, t.g, pb, nb);
    }
    G64 dst;
    if (d.arity) {
      dst = vals + t.g * d.arity;
    } else {
      const uint32_t c = d.kind == OP_CROSS ? na * nb : na + nb;
      dst = vals + place_ragged(P, t, d, c);
    }
    if (!t.live) continue;
    if (d.kind == OP_CROSS) {
      for (uint32_t i = 0; i < na; ++i) {
        const uint64_t ma = mix64(pa[i] + d.key);
        for (uint32_t j = 0; j < nb; ++j) *dst++ = mix64(ma + pb[j]);
      }
    } else {
      for (uint32_t i = 0; i < na; ++i) *dst++ = pa[i];
      for (uint32_t j = 0; j < nb; ++j) *dst++ = pb[j];
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_walk(WalkParams P) {
  if (P.ctrl->err) return;  // an earlier kernel of this call found a problem
  Tile t;
  if (!tile_of_wave(P.n_tiles, kBlock / 64, t.tile)) return;
  open_tile(P, t, P.layer_lo == 1, (threadIdx.x >> 6) * kRingWave);
  uint32_t malformed = 0;
  for (uint32_t layer = P.layer_lo; layer <= P.layer_hi; ++layer) {
    if (layer == 1) walk_roots(P, t, malformed);
    else run_layer(P, t, layer);
    // a lane reads back only what this wavefront stored; make those stores land first
    if (layer < P.layer_hi) __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  }
  const uint64_t wm = wave_sum64(malformed);
  if (lane_id() == 0 && wm) atomicAdd(reinterpret_cast<unsigned long long*>(&P.ctrl->n_malformed), (unsigned long long)wm);
}

// ----------------------------------------------------------- launch wrappers
static dim3 tile_grid(uint32_t n_tiles, uint32_t waves_per_block) {
  const uint32_t blocks = (n_tiles + waves_per_block - 1) / waves_per_block;
  return dim3(((blocks + 7u) / 8u) * 8u);
}

hipError_t launch_count(const WalkParams& P, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  const uint32_t lds = std::max(P.waves_per_block * (kRingWave + P.n_ragged * 64u) * (uint32_t)sizeof(uint32_t), P.lds_pad);
  if (lds > 64u * 1024u) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_count),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_count, tile_grid(P.n_tiles, P.waves_per_block), dim3(P.waves_per_block * 64u), lds, st, P);
  return hipGetLastError();
}

hipError_t launch_walk(const WalkParams& P, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  hipLaunchKernelGGL(k_walk, tile_grid(P.n_tiles, kBlock / 64), dim3(kBlock),
                     std::max((uint32_t)((kBlock / 64) * kRingWave * sizeof(uint32_t)), P.lds_pad), st, P);
  return hipGetLastError();
}

}  // namespace fbx
