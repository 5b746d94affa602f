// HIP kernels of libfbx for gfx950 (MI355X) and their launch wrappers.
//
// Work decomposition.  Records are independent (every operator computes on one
// row of the table; Section 3, "Extract features"), so the batch is cut into
// tiles of T consecutive records (T a power of two, at most 64) and one
// workgroup of four wavefronts owns one tile.  The workgroup stages the tile's
// raw bytes in LDS with coalesced 16-byte loads, finds every tab while the
// bytes pass through registers, and then evaluates the operators of a layer
// with lanes running over (record, operator) pairs, records fastest, so that
// stores to a slot's value array are contiguous across lanes.
//
// Variable-length outputs.  The paper hands out dynamic memory with one atomic
// add per thread block (Section 5, Algorithm 1), which places blocks in
// arrival order.  A record-ordered CSR needs ordered placement instead, so a
// first pass over the tiles only counts, a scan turns the per-tile counts into
// per-tile bases, Algorithm 1 is then used once, on the device, to carve the
// operators' arrays out of the pool, and the second pass writes.
#include <hip/hip_runtime.h>

#include "fbx_device.h"

namespace fbx {

constexpr int kWaves = kBlock / 64;
constexpr uint32_t kNoRow = 0xffffffffu;
constexpr uint64_t kPrime = 0x100000001b3ull;

extern __shared__ __align__(16) uint8_t smem[];

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

// Tab bits of one little-endian dword: bit j set iff byte j == '\t'.
__device__ __forceinline__ uint32_t tab_bits(uint32_t w) {
  uint32_t x = w ^ 0x09090909u;
  uint32_t m = ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);  // 0x80 in every zero byte
  return (((m >> 7) * 0x00204081u) >> 21) & 0xfu;
}

// Byte sources: a tile staged in LDS (fast path) or read in place (slow path).
// Indices are relative to the first byte of the tile.
struct LdsSrc {
  uint32_t base;  // offset of tile byte 0 inside smem
  __device__ __forceinline__ uint32_t at(uint32_t i) const { return smem[base + i]; }
};
struct GlbSrc {
  const uint8_t* p;  // address of tile byte 0
  __device__ __forceinline__ uint32_t at(uint32_t i) const { return p[i]; }
};

// Per-tile record framing kept in LDS.
struct Frame {
  uint32_t rec_start[65];
  uint32_t rec_end[64];
  uint32_t rec_tab[65];
};

// Field k of record r: the bytes between its k-th and (k+1)-th tab; records
// with fewer tabs have empty trailing fields.
template <bool FAST, class Src>
__device__ __forceinline__ void field_span(const Frame& fr, const uint16_t* tabpos, const Src& S, uint32_t r,
                                           uint32_t k, uint32_t& s, uint32_t& e) {
  const uint32_t rs = fr.rec_start[r], re = fr.rec_end[r];
  if (FAST) {
    const uint32_t t0 = fr.rec_tab[r], nt = fr.rec_tab[r + 1] - t0;
    if (k > nt) { s = e = re; return; }
    s = k == 0 ? rs : (uint32_t)tabpos[t0 + k - 1] + 1u;
    e = k < nt ? (uint32_t)tabpos[t0 + k] : re;
  } else {
    uint32_t pos = rs;
    for (uint32_t f = 0; f < k; ++f) {
      while (pos < re && S.at(pos) != '\t') ++pos;
      if (pos == re) { s = e = re; return; }
      ++pos;
    }
    uint32_t end = pos;
    while (end < re && S.at(end) != '\t') ++end;
    s = pos; e = end;
  }
}

template <class Src>
__device__ __forceinline__ bool starts_with(const Src& S, uint32_t s, uint32_t e, const uint8_t* pre, uint32_t plen) {
  if (e - s < plen) return false;
  for (uint32_t j = 0; j < plen; ++j)
    if (S.at(s + j) != pre[j]) return false;
  return true;
}

// Number of signs a root operator produces for the field [s, e).
template <class Src>
__device__ uint32_t root_count(const OpDesc& d, const uint8_t* aux, const Src& S, uint32_t s, uint32_t e) {
  switch (d.kind) {
    case OP_HASH:
    case OP_BUCKET: {
      if (!(d.flags & F_MULTI)) return 1;
      uint32_t c = 1;
      for (uint32_t i = s; i < e; ++i) c += S.at(i) == ',';
      return c;
    }
    case OP_NGRAM: {
      const uint32_t L = e - s, n = d.aux_len;
      return L >= n ? L - n + 1 : 0;
    }
    case OP_FILTER: {
      const uint8_t* pre = aux + d.aux_off;
      if (!(d.flags & F_MULTI)) return starts_with(S, s, e, pre, d.aux_len) ? 1u : 0u;
      uint32_t c = 0, t0 = s;
      for (uint32_t i = s; i <= e; ++i)
        if (i == e || S.at(i) == ',') {
          c += starts_with(S, t0, i, pre, d.aux_len) ? 1u : 0u;
          t0 = i + 1;
        }
      return c;
    }
    default:
      return 0;
  }
}

// Decimal text [t0, t1) -> signed micro-units; sets bad when the text is not
// entirely of the form -?digits*(.digits*)? with at least one digit.
template <class Src>
__device__ __forceinline__ int64_t parse_micro(const Src& S, uint32_t t0, uint32_t t1, bool& bad) {
  uint32_t i = t0;
  bool neg = false;
  if (i < t1 && S.at(i) == '-') { neg = true; ++i; }
  uint64_t ip = 0, fp = 0;
  uint32_t digits = 0, nfrac = 0;
  while (i < t1) {
    uint32_t c = S.at(i) - '0';
    if (c > 9) break;
    ip = ip * 10u + c; ++digits; ++i;
  }
  if (i < t1 && S.at(i) == '.') {
    ++i;
    while (i < t1) {
      uint32_t c = S.at(i) - '0';
      if (c > 9) break;
      if (nfrac < 6) { fp = fp * 10u + c; ++nfrac; }
      ++digits; ++i;
    }
  }
  for (; nfrac < 6; ++nfrac) fp *= 10u;
  uint64_t v = ip * 1000000ull + fp;
  if (neg) v = 0ull - v;
  bad = (i < t1) || digits == 0;
  return (int64_t)v;
}

template <class Src>
__device__ __forceinline__ uint64_t bucket_sign(const OpDesc& d, const uint8_t* aux, const Src& S, uint32_t t0,
                                                uint32_t t1, uint32_t& malformed) {
  bool bad;
  const int64_t v = parse_micro(S, t0, t1, bad);
  malformed += bad ? 1u : 0u;
  const int64_t* b = reinterpret_cast<const int64_t*>(aux + d.aux_off);
  uint32_t lo = 0, hi = d.aux_len;  // index = number of boundaries <= v
  while (lo < hi) {
    uint32_t mid = (lo + hi) >> 1;
    if (b[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return mix64(d.key + lo);
}

// Signs of a root operator (not n-gram) for the field [s, e), written to out[0..count).
template <class Src>
__device__ void root_emit(const OpDesc& d, const uint8_t* aux, const Src& S, uint32_t s, uint32_t e, uint64_t* out,
                          uint32_t& malformed) {
  const bool multi = d.flags & F_MULTI;
  switch (d.kind) {
    case OP_HASH: {
      uint64_t h = d.key;
      uint32_t j = 0;
      for (uint32_t i = s; i < e; ++i) {
        uint32_t c = S.at(i);
        if (multi && c == ',') { out[j++] = h; h = d.key; }
        else h = (h ^ c) * kPrime;
      }
      out[j] = h;
      break;
    }
    case OP_FILTER: {
      const uint8_t* pre = aux + d.aux_off;
      const uint32_t plen = d.aux_len;
      uint64_t h = d.key;
      uint32_t j = 0, k = 0;
      bool match = true;
      for (uint32_t i = s; i <= e; ++i) {
        uint32_t c = i < e ? S.at(i) : 0x100u;
        if (i == e || (multi && c == ',')) {
          if (match && k >= plen) out[j++] = h;
          h = d.key; k = 0; match = true;
        } else {
          if (k < plen && c != pre[k]) match = false;
          h = (h ^ c) * kPrime;
          ++k;
        }
      }
      break;
    }
    case OP_BUCKET: {
      if (!multi) { out[0] = bucket_sign(d, aux, S, s, e, malformed); break; }
      uint32_t j = 0, t0 = s;
      for (uint32_t i = s; i <= e; ++i)
        if (i == e || S.at(i) == ',') {
          out[j++] = bucket_sign(d, aux, S, t0, i, malformed);
          t0 = i + 1;
        }
      break;
    }
    default:
      break;
  }
}

// Length and address of an operator's list for global record g.
__device__ __forceinline__ void input_list(const TileParams& P, uint32_t op, uint64_t g, const uint64_t*& ptr,
                                           uint64_t& n) {
  const OpDesc& d = P.ops[op];
  const OpDyn& y = P.dyn[op];
  const uint64_t* vals = reinterpret_cast<const uint64_t*>(P.ws + y.values_off);
  if (d.arity) {
    n = d.arity;
    ptr = vals + g * d.arity;
  } else {
    const uint64_t* off = reinterpret_cast<const uint64_t*>(P.ws + y.offsets_off);
    const uint64_t o0 = off[g], o1 = off[g + 1];
    n = o1 - o0;
    ptr = vals + o0;
  }
}

// ------------------------------------------------------------ tile framing
// Stage the tile into LDS, build the tab list and the per-record framing.
// Returns true when the tile fits the fast path.
__device__ bool stage_tile(const TileParams& P, Frame& fr, uint32_t* s_misc, uint64_t tile_lo, uint32_t nbytes,
                           uint32_t Tn) {
  const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const uint8_t* src = P.raw + tile_lo;
  const uint32_t head = (uint32_t)(reinterpret_cast<uintptr_t>(src) & 15u);
  uint8_t* bytes = smem + P.lds_bytes;
  uint16_t* mask16 = reinterpret_cast<uint16_t*>(smem + P.lds_mask);
  uint16_t* tabpos = reinterpret_cast<uint16_t*>(smem + P.lds_tab);
  if ((uint64_t)nbytes + head > P.cap_bytes) return false;  // block-uniform

  const uint8_t* abase = src - head;  // 16-byte aligned; may lie before raw
  const uint8_t* raw_end = P.raw + P.raw_len;
  const uint32_t span = head + nbytes;
  const uint32_t npieces = (span + 15u) >> 4;
  const uint32_t per_wave = (((npieces + kWaves - 1) / kWaves) + 63u) & ~63u;
  const uint32_t p_lo = wave * per_wave;
  const uint32_t p_hi = min(p_lo + per_wave, npieces);

  uint32_t my_tabs = 0;
  for (uint32_t p = p_lo + lane; p < p_hi; p += 64) {
    const uint8_t* a = abase + (uint64_t)p * 16u;
    uint4 v;
    if (a >= P.raw && a + 16 <= raw_end) {
      v = *reinterpret_cast<const uint4*>(a);
    } else {
      uint32_t w[4] = {0, 0, 0, 0};
      for (int j = 0; j < 16; ++j)
        if (a + j >= P.raw && a + j < raw_end) w[j >> 2] |= (uint32_t)a[j] << (8 * (j & 3));
      v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    *reinterpret_cast<uint4*>(bytes + p * 16u) = v;
    uint32_t m = tab_bits(v.x) | (tab_bits(v.y) << 4) | (tab_bits(v.z) << 8) | (tab_bits(v.w) << 12);
    // keep only bytes that belong to this tile
    const uint32_t first = p * 16u;
    const uint32_t lo = head > first ? head - first : 0u;
    const uint32_t hi = span - first < 16u ? span - first : 16u;
    m &= (0xffffu << lo) & (0xffffu >> (16u - hi));
    mask16[p] = (uint16_t)m;
    my_tabs += __popc(m);
  }
  const uint32_t wave_tabs = (uint32_t)wave_sum64(my_tabs);
  if (lane == 0) s_misc[wave] = wave_tabs;
  __syncthreads();
  uint32_t base = 0, total = 0;
  for (int w = 0; w < kWaves; ++w) {
    if ((uint32_t)w < wave) base += s_misc[w];
    total += s_misc[w];
  }
  const bool fits = total <= P.cap_tabs;  // block-uniform
  if (fits) {
    for (uint32_t p0 = p_lo; p0 < p_hi; p0 += 64) {
      const uint32_t p = p0 + lane;
      uint32_t m = p < p_hi ? mask16[p] : 0u;
      const uint32_t c = __popc(m);
      const uint32_t incl = wave_incl_scan(c);
      uint32_t idx = base + incl - c;
      while (m) {
        const uint32_t bit = __ffs(m) - 1;
        tabpos[idx++] = (uint16_t)(p * 16u + bit - head);
        m &= m - 1;
      }
      base += __shfl(incl, 63, 64);
    }
  }
  __syncthreads();
  if (!fits) return false;
  // tab index at the start of every record (tab positions are sorted)
  if (tid <= Tn) {
    const uint32_t key = fr.rec_start[tid];
    uint32_t lo = 0, hi = total;
    while (lo < hi) {
      uint32_t mid = (lo + hi) >> 1;
      if ((uint32_t)tabpos[mid] < key) lo = mid + 1; else hi = mid;
    }
    fr.rec_tab[tid] = lo;
  }
  return true;
}

// ------------------------------------------------------------------ layers
template <bool FAST, class Src>
__device__ void count_tile(const TileParams& P, const Frame& fr, const Src& S, uint32_t tile, uint32_t Tn) {
  const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const uint32_t T = 1u << P.log2T;
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem + P.lds_cnt);
  const uint16_t* tabpos = reinterpret_cast<const uint16_t*>(smem + P.lds_tab);
  const uint32_t l0 = P.layer_begin[0], nl = P.layer_begin[1] - l0;
  for (uint32_t item = tid; item < (nl << P.log2T); item += kBlock) {
    const uint32_t r = item & (T - 1), oi = item >> P.log2T;
    if (r >= Tn) continue;
    const OpDesc& d = P.ops[P.layer_ops[l0 + oi]];
    if (d.rag_row == kNoRow) continue;
    uint32_t s, e;
    field_span<FAST>(fr, tabpos, S, r, d.field, s, e);
    cnt[d.rag_row * T + r] = root_count(d, P.aux, S, s, e);
  }
  __syncthreads();
  // counts of the later layers follow from the inputs' counts, record by record
  if (tid < Tn) {
    bool overflow = false;
    for (uint32_t k = 0; k < P.n_nonroot; ++k) {
      const OpDesc& d = P.ops[P.nonroot[k]];
      if (d.rag_row == kNoRow) continue;
      const OpDesc& da = P.ops[d.a];
      const OpDesc& db = P.ops[d.b];
      const uint64_t ca = da.arity ? da.arity : cnt[da.rag_row * T + tid];
      const uint64_t cb = db.arity ? db.arity : cnt[db.rag_row * T + tid];
      const uint64_t c = d.kind == OP_CROSS ? ca * cb : ca + cb;
      if (c > 0x7fffffffull) overflow = true;
      cnt[d.rag_row * T + tid] = (uint32_t)c;
    }
    if (overflow) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
  }
  __syncthreads();
  for (uint32_t row = wave; row < P.n_ragged; row += kWaves) {
    uint64_t v = lane < Tn ? cnt[row * T + lane] : 0u;
    v = wave_sum64(v);
    if (lane == 0) {
      if (v > 0x7fffffffull) atomicOr(&P.ctrl->err, (uint32_t)CE_OVERFLOW);
      P.tile_cnt[(uint64_t)row * P.n_tiles + tile] = (uint32_t)v;
    }
  }
}

template <bool FAST, class Src>
__device__ void write_tile(const TileParams& P, const Frame& fr, const Src& S, uint32_t tile, uint64_t g0,
                           uint32_t Tn) {
  const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const uint32_t T = 1u << P.log2T;
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem + P.lds_cnt);
  const uint16_t* tabpos = reinterpret_cast<const uint16_t*>(smem + P.lds_tab);
  uint32_t malformed = 0;

  for (uint32_t layer = P.layer_lo; layer <= P.layer_hi; ++layer) {
    const uint32_t l0 = P.layer_begin[layer - 1], nl = P.layer_begin[layer] - l0;
    const uint32_t n_items = nl << P.log2T;
    // pass A: per-record counts of the ragged operators of this layer
    for (uint32_t item = tid; item < n_items; item += kBlock) {
      const uint32_t r = item & (T - 1), oi = item >> P.log2T;
      if (r >= Tn) continue;
      const OpDesc& d = P.ops[P.layer_ops[l0 + oi]];
      if (d.rag_row == kNoRow) continue;
      uint32_t c;
      if (layer == 1) {
        uint32_t s, e;
        field_span<FAST>(fr, tabpos, S, r, d.field, s, e);
        c = root_count(d, P.aux, S, s, e);
      } else {
        const uint64_t* pa; const uint64_t* pb; uint64_t na, nb;
        input_list(P, d.a, g0 + r, pa, na);
        input_list(P, d.b, g0 + r, pb, nb);
        c = (uint32_t)(d.kind == OP_CROSS ? na * nb : na + nb);
      }
      cnt[d.rag_row * T + r] = c;
    }
    __syncthreads();
    // in-tile exclusive prefix per ragged operator (one wavefront per operator),
    // shifted by the tile's base: these are the CSR offsets of the tile's records
    for (uint32_t oi = wave; oi < nl; oi += kWaves) {
      const uint32_t op = P.layer_ops[l0 + oi];
      const OpDesc& d = P.ops[op];
      if (d.rag_row == kNoRow) continue;
      const uint32_t c = lane < Tn ? cnt[d.rag_row * T + lane] : 0u;
      const uint32_t incl = wave_incl_scan(c);
      const uint64_t base = P.tile_base[(uint64_t)d.rag_row * P.n_tiles + tile];
      uint64_t* off = reinterpret_cast<uint64_t*>(P.ws + P.dyn[op].offsets_off);
      if (lane < Tn) {
        cnt[d.rag_row * T + lane] = incl - c;
        off[g0 + lane] = base + (incl - c);
        // the entry after the tile's last record equals the next tile's first
        // entry; writing it here too keeps a tile's view of its own offsets complete
        if (lane == Tn - 1) off[g0 + Tn] = base + incl;
      }
    }
    __syncthreads();
    // pass B: values
    for (uint32_t item = tid; item < n_items; item += kBlock) {
      const uint32_t r = item & (T - 1), oi = item >> P.log2T;
      if (r >= Tn) continue;
      const uint32_t op = P.layer_ops[l0 + oi];
      const OpDesc& d = P.ops[op];
      if (d.kind == OP_NGRAM) continue;
      uint64_t* vals = reinterpret_cast<uint64_t*>(P.ws + P.dyn[op].values_off);
      uint64_t* dst;
      if (d.arity) dst = vals + (g0 + r) * d.arity;
      else dst = vals + P.tile_base[(uint64_t)d.rag_row * P.n_tiles + tile] + cnt[d.rag_row * T + r];
      if (layer == 1) {
        uint32_t s, e;
        field_span<FAST>(fr, tabpos, S, r, d.field, s, e);
        root_emit(d, P.aux, S, s, e, dst, malformed);
      } else {
        const uint64_t* pa; const uint64_t* pb; uint64_t na, nb;
        input_list(P, d.a, g0 + r, pa, na);
        input_list(P, d.b, g0 + r, pb, nb);
        if (d.kind == OP_CROSS) {
          for (uint64_t i = 0; i < na; ++i) {
            const uint64_t ma = mix64(pa[i] + d.key);
            for (uint64_t j = 0; j < nb; ++j) *dst++ = mix64(ma + pb[j]);
          }
        } else {
          for (uint64_t i = 0; i < na; ++i) *dst++ = pa[i];
          for (uint64_t j = 0; j < nb; ++j) *dst++ = pb[j];
        }
      }
    }
    // n-grams: one wavefront per record, lanes over the grams
    if (layer == 1) {
      for (uint32_t oi = 0; oi < nl; ++oi) {
        const uint32_t op = P.layer_ops[l0 + oi];
        const OpDesc& d = P.ops[op];
        if (d.kind != OP_NGRAM) continue;
        uint64_t* vals = reinterpret_cast<uint64_t*>(P.ws + P.dyn[op].values_off);
        const uint64_t base = P.tile_base[(uint64_t)d.rag_row * P.n_tiles + tile];
        const uint32_t n = d.aux_len;
        for (uint32_t r = wave; r < Tn; r += kWaves) {
          uint32_t s, e;
          field_span<FAST>(fr, tabpos, S, r, d.field, s, e);
          const uint32_t L = e - s;
          const uint32_t ng = L >= n ? L - n + 1 : 0;
          uint64_t* dst = vals + base + cnt[d.rag_row * T + r];
          for (uint32_t k = lane; k < ng; k += 64) {
            uint64_t h = d.key;
            for (uint32_t j = 0; j < n; ++j) h = (h ^ S.at(s + k + j)) * kPrime;
            dst[k] = h;
          }
        }
      }
    }
    if (layer < P.layer_hi) {
      __threadfence();
      __syncthreads();
    }
  }
  const uint64_t wm = wave_sum64(malformed);
  if (lane == 0 && wm) atomicAdd(reinterpret_cast<unsigned long long*>(&P.ctrl->n_malformed), (unsigned long long)wm);
}

template <bool COUNT>
__global__ __launch_bounds__(kBlock) void k_tile(TileParams P) {
  __shared__ Frame fr;
  __shared__ uint32_t s_misc[8];
  if (P.ctrl->err) return;  // an earlier kernel of this call found a problem
  // Consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each
  // XCD a contiguous run of tiles so that neighbouring tiles share an L2.
  const uint32_t chunk = (P.n_tiles + 7u) >> 3;
  const uint32_t tile = (blockIdx.x & 7u) * chunk + (blockIdx.x >> 3);
  if (tile >= P.n_tiles) return;
  const uint32_t tid = threadIdx.x;
  const uint64_t g0 = (uint64_t)tile << P.log2T;
  const uint64_t left = P.n_records - g0;
  const uint32_t Tn = left < (1ull << P.log2T) ? (uint32_t)left : (1u << P.log2T);
  const bool need_raw = COUNT || P.layer_lo == 1;
  bool fast = false;
  uint64_t tile_lo = 0;
  if (need_raw) {
    tile_lo = P.rec_off[g0];
    const uint64_t tile_hi = P.rec_off[g0 + Tn];
    if (tid <= Tn) fr.rec_start[tid] = (uint32_t)(P.rec_off[g0 + tid] - tile_lo);
    __syncthreads();
    fast = stage_tile(P, fr, s_misc, tile_lo, (uint32_t)(tile_hi - tile_lo), Tn);
    if (!fast && tid == 0) atomicAdd(reinterpret_cast<unsigned long long*>(&P.ctrl->slow_tiles), 1ull);
    // one trailing newline is not part of the record
    if (tid < Tn) {
      const uint32_t s = fr.rec_start[tid];
      uint32_t e = fr.rec_start[tid + 1];
      if (e > s && P.raw[tile_lo + e - 1] == '\n') --e;
      fr.rec_end[tid] = e;
    }
    __syncthreads();
  }
  if (fast) {
    const uint32_t head = (uint32_t)(reinterpret_cast<uintptr_t>(P.raw + tile_lo) & 15u);
    LdsSrc S{P.lds_bytes + head};
    if (COUNT) count_tile<true>(P, fr, S, tile, Tn);
    else write_tile<true>(P, fr, S, tile, g0, Tn);
  } else {
    GlbSrc S{P.raw + tile_lo};
    if (COUNT) count_tile<false>(P, fr, S, tile, Tn);
    else write_tile<false>(P, fr, S, tile, g0, Tn);
  }
}

// --------------------------------------------------------------- validation
__global__ void k_reset(Ctrl* ctrl, uint64_t arena_base) {
  if (threadIdx.x == 0) {
    ctrl->err = 0; ctrl->pad0 = 0; ctrl->required = 0; ctrl->head = arena_base; ctrl->high_water = arena_base;
    ctrl->n_malformed = 0; ctrl->max_tile_bytes = 0; ctrl->slow_tiles = 0; ctrl->pad1 = 0;
  }
}

__global__ void k_validate(const uint64_t* rec_off, uint64_t n_records, uint64_t raw_len, uint32_t log2T, Ctrl* ctrl) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_records) return;
  const uint64_t a = rec_off[i], b = rec_off[i + 1];
  uint32_t err = 0;
  if (a > b || b > raw_len) err |= CE_OFFSETS;
  if ((i & ((1ull << log2T) - 1)) == 0) {
    const uint64_t j = i + (1ull << log2T) < n_records ? i + (1ull << log2T) : n_records;
    const uint64_t hi = rec_off[j];
    if (hi >= a) {
      if (hi - a >= (1ull << 31)) err |= CE_TILE;
      atomicMax(reinterpret_cast<unsigned long long*>(&ctrl->max_tile_bytes), (unsigned long long)(hi - a));
    }
  }
  if (err) atomicOr(&ctrl->err, err);
}

// --------------------------------------------------------------------- scan
// Exclusive scan over tiles of one ragged operator's per-tile counts.
__global__ __launch_bounds__(kBlock) void k_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total,
                                                 uint32_t n_tiles, const Ctrl* ctrl) {
  __shared__ uint64_t s[kBlock];
  if (ctrl->err) return;
  const uint32_t row = blockIdx.x, tid = threadIdx.x;
  const uint32_t* src = tile_cnt + (uint64_t)row * n_tiles;
  uint64_t* dst = tile_base + (uint64_t)row * n_tiles;
  const uint32_t chunk = (n_tiles + kBlock - 1) / kBlock;
  const uint32_t lo = min(tid * chunk, n_tiles), hi = min(lo + chunk, n_tiles);
  uint64_t sum = 0;
  for (uint32_t i = lo; i < hi; ++i) sum += src[i];
  s[tid] = sum;
  __syncthreads();
  for (int d = 1; d < kBlock; d <<= 1) {
    uint64_t t = tid >= (uint32_t)d ? s[tid - d] : 0;
    __syncthreads();
    s[tid] += t;
    __syncthreads();
  }
  uint64_t run = s[tid] - sum;
  for (uint32_t i = lo; i < hi; ++i) { dst[i] = run; run += src[i]; }
  if (tid == kBlock - 1) row_total[row] = s[tid];
}

// ------------------------------------------------------------------- arena
__device__ __forceinline__ uint64_t round128(uint64_t x) { return (x + 127ull) & ~127ull; }

// Algorithm 1 of the paper (Section 5): every thread of the block brings a
// size; the block takes a prefix sum, ONE thread adds the block's total to the
// idle-memory head with an atomic add, and every thread's offset is the old
// head plus the sizes of the threads before it.  (The listing subtracts the
// first thread's prefix, which is only right for equal sizes; the prose and
// the figure call for the exclusive prefix, which is what is computed here.)
// The block total is rounded up to 128 bytes so that every block starts on a
// 128-byte line, as the paper asks.  s_scan must hold blockDim.x entries.
__device__ uint64_t arena_alloc_block(uint64_t* head, uint64_t size, uint64_t* s_scan, uint64_t* s_addr) {
  const uint32_t tid = threadIdx.x, n = blockDim.x;
  s_scan[tid] = size;
  __syncthreads();
  for (uint32_t d = 1; d < n; d <<= 1) {
    uint64_t t = tid >= d ? s_scan[tid - d] : 0;
    __syncthreads();
    s_scan[tid] += t;
    __syncthreads();
  }
  const uint64_t incl = s_scan[tid];
  if (tid == 0) {
    const uint64_t total = round128(s_scan[n - 1]);
    *s_addr = total ? atomicAdd(reinterpret_cast<unsigned long long*>(head), (unsigned long long)total)
                    : *reinterpret_cast<volatile uint64_t*>(head);
  }
  __syncthreads();
  const uint64_t out = *s_addr + incl - size;
  __syncthreads();
  return out;
}

__global__ void k_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets) {
  extern __shared__ __align__(16) uint8_t dyn_smem[];
  uint64_t* s_scan = reinterpret_cast<uint64_t*>(dyn_smem);
  __shared__ uint64_t s_addr;
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t size = i < n ? sizes[i] : 0;
  const uint64_t off = arena_alloc_block(head, size, s_scan, &s_addr);
  if (i < n) offsets[i] = off;
}

__global__ void k_arena_reset(uint64_t* head, uint64_t value) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *head = value;
}

// Carve the operators' value / offset arrays out of the pool, once sizes are
// known.  Emitted operators first (they live until the next call); then layer
// by layer the intermediates born in that layer, and after each layer the head
// drops back as far as still-live intermediates allow: the constant-time reset
// of Section 5 ("Reset GPU memory pool"), generalised to outputs that a later
// layer still reads.  With reuse off (all layers in one launch) nothing is
// released.  One block of kBlock threads.
__global__ __launch_bounds__(kBlock) void k_alloc(const OpDesc* ops, OpDyn* dyn, uint32_t n_ops, uint32_t n_layers,
                                                  const uint64_t* row_total, uint64_t n_records, uint64_t ws_bytes,
                                                  uint8_t* ws, int reuse, Ctrl* ctrl) {
  __shared__ uint64_t s_scan[kBlock];
  __shared__ uint64_t s_addr;
  __shared__ unsigned long long s_max;
  if (ctrl->err) return;
  const uint32_t tid = threadIdx.x;
  uint64_t high = ctrl->head;
  uint64_t persist_end = high;  // end of the emitted operators' storage
  for (uint32_t pass = 0; pass <= n_layers; ++pass) {  // pass 0: emitted; pass l: intermediates of layer l
    for (uint32_t c0 = 0; c0 < n_ops; c0 += kBlock) {
      const uint32_t i = c0 + tid;
      uint64_t sv = 0, so = 0, nv = 0;
      bool mine = false;
      if (i < n_ops) {
        const OpDesc& d = ops[i];
        const bool emit = d.flags & F_EMIT;
        mine = pass == 0 ? emit : (!emit && d.layer == pass);
        if (mine) {
          nv = d.arity ? n_records * d.arity : row_total[d.rag_row];
          sv = round128(nv * 8ull);
          so = d.arity ? 0 : round128((n_records + 1) * 8ull);
        }
      }
      const uint64_t off = arena_alloc_block(&ctrl->head, sv + so, s_scan, &s_addr);
      if (mine) {
        dyn[i].values_off = off;
        dyn[i].offsets_off = so ? off + sv : 0;
        dyn[i].n_values = nv;
        dyn[i].pad = off + sv + so;  // end of this operator's storage
      }
    }
    __threadfence();
    __syncthreads();
    const uint64_t head_now = *reinterpret_cast<volatile uint64_t*>(&ctrl->head);
    if (head_now > high) high = head_now;
    if (pass == 0) persist_end = head_now;
    if (pass >= 1 && reuse) {
      // release: the head drops to the end of the highest still-live intermediate
      if (tid == 0) s_max = persist_end;
      __syncthreads();
      unsigned long long m = 0;
      for (uint32_t i = tid; i < n_ops; i += kBlock) {
        const OpDesc& d = ops[i];
        if (!(d.flags & F_EMIT) && d.layer <= pass && d.death > pass) m = max(m, (unsigned long long)dyn[i].pad);
      }
      atomicMax(&s_max, m);
      __syncthreads();
      if (tid == 0) *reinterpret_cast<volatile uint64_t*>(&ctrl->head) = s_max;
      __threadfence();
      __syncthreads();
    }
  }
  if (tid == 0) {
    ctrl->high_water = high;
    ctrl->required = high;
    if (high > ws_bytes) atomicOr(&ctrl->err, (uint32_t)CE_NOMEM);
  }
  // an empty batch still owes every ragged slot its single offset entry
  if (n_records == 0 && high <= ws_bytes) {
    for (uint32_t i = tid; i < n_ops; i += kBlock)
      if (!ops[i].arity) *reinterpret_cast<uint64_t*>(ws + dyn[i].offsets_off) = 0;
  }
}

// ----------------------------------------------------------- launch wrappers
hipError_t launch_reset(Ctrl* ctrl, uint64_t arena_base, hipStream_t st) {
  hipLaunchKernelGGL(k_reset, dim3(1), dim3(64), 0, st, ctrl, arena_base);
  return hipGetLastError();
}

hipError_t launch_validate(const uint64_t* rec_off, uint64_t n_records, uint64_t raw_len, uint32_t log2T, Ctrl* ctrl,
                           hipStream_t st) {
  if (n_records == 0) return hipSuccess;
  const uint64_t blocks = (n_records + 255) / 256;
  hipLaunchKernelGGL(k_validate, dim3((uint32_t)blocks), dim3(256), 0, st, rec_off, n_records, raw_len, log2T, ctrl);
  return hipGetLastError();
}

hipError_t launch_tile(const TileParams& P, bool count, uint32_t lds_bytes, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tile<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tile<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048);
    if (e != hipSuccess) (void)hipGetLastError();  // only needed above 64 KB; launch will report if it matters
    attr_done = true;
  }
  const uint32_t chunk = (P.n_tiles + 7u) / 8u;
  const dim3 grid(chunk * 8u);
  if (count) hipLaunchKernelGGL(k_tile<true>, grid, dim3(kBlock), lds_bytes, st, P);
  else hipLaunchKernelGGL(k_tile<false>, grid, dim3(kBlock), lds_bytes, st, P);
  return hipGetLastError();
}

hipError_t launch_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total, uint32_t n_ragged,
                       uint32_t n_tiles, const Ctrl* ctrl, hipStream_t st) {
  if (n_ragged == 0) return hipSuccess;
  hipLaunchKernelGGL(k_scan, dim3(n_ragged), dim3(kBlock), 0, st, tile_cnt, tile_base, row_total, n_tiles, ctrl);
  return hipGetLastError();
}

hipError_t launch_alloc(const OpDesc* ops, OpDyn* dyn, uint32_t n_ops, uint32_t n_layers, const uint64_t* row_total,
                        uint64_t n_records, uint64_t ws_bytes, uint8_t* ws, int reuse, Ctrl* ctrl, hipStream_t st) {
  hipLaunchKernelGGL(k_alloc, dim3(1), dim3(kBlock), 0, st, ops, dyn, n_ops, n_layers, row_total, n_records, ws_bytes,
                     ws, reuse, ctrl);
  return hipGetLastError();
}

hipError_t launch_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets, uint32_t threads,
                              hipStream_t st) {
  if (n == 0) return hipSuccess;
  const uint64_t blocks = (n + threads - 1) / threads;
  hipLaunchKernelGGL(k_arena_alloc, dim3((uint32_t)blocks), dim3(threads), threads * sizeof(uint64_t), st, head, sizes,
                     n, offsets);
  return hipGetLastError();
}

hipError_t launch_arena_reset(uint64_t* head, uint64_t value, hipStream_t st) {
  hipLaunchKernelGGL(k_arena_reset, dim3(1), dim3(64), 0, st, head, value);
  return hipGetLastError();
}

}  // namespace fbx
