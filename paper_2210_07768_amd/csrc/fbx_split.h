// Splitting staged bytes at a delimiter with groups of lanes (Section 5 of the paper, first
// paragraph: a record is split at its delimiter before anything else happens to it), shared by the
// tile kernel of the extraction path and by the cleaning stage.  Device code for gfx950 only.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace fbx {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The thread's number, hidden from the optimiser's view of the loops around the caller: what
// follows from it (lane masks, per-lane addresses) is then worked out where it is used instead
// of once per kernel, where each such value would hold a register for good.
__device__ __forceinline__ uint32_t thread_id() {
  uint32_t t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}
__device__ __forceinline__ uint32_t lane_id() { return thread_id() & 63u; }

// 0x80 in exactly the bytes of w that equal the byte repeated in pat.
__device__ __forceinline__ uint32_t eq_flags(uint32_t w, uint32_t pat) {
  const uint32_t x = w ^ pat;
  return ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);
}
constexpr uint32_t kTabs = 0x09090909u, kCommas = 0x2c2c2c2cu;

// Inclusive prefix sum of v inside groups of 1 << lg neighbouring lanes (j: the lane's number in
// its group).  Inside a row of 16 lanes the steps of 1, 2, 4 and 8 lanes are single
// data-parallel-primitive moves (row_shr, zero for a lane without a source); a group of several
// rows then adds the totals of its earlier rows, which come through the LDS crossbar.  Every
// lane of the wavefront must call it.
template <int D>
__device__ __forceinline__ uint32_t row_shr(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x110 + D, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t group_prefix(uint32_t v, uint32_t lg, uint32_t j) {
  if (lg >= 1u) { const uint32_t t = row_shr<1>(v); v += j >= 1u ? t : 0u; }
  if (lg >= 2u) { const uint32_t t = row_shr<2>(v); v += j >= 2u ? t : 0u; }
  if (lg >= 3u) { const uint32_t t = row_shr<4>(v); v += j >= 4u ? t : 0u; }
  if (lg >= 4u) { const uint32_t t = row_shr<8>(v); v += j >= 8u ? t : 0u; }
  if (lg > 4u) {  // groups of two or four rows: add the totals of the group's rows before the lane's own
    const uint32_t first = lane_id() - j;
    uint32_t carry = 0;
    for (uint32_t k = 1; k < (1u << (lg - 4u)); ++k) {
      const uint32_t t = __shfl(v, (int)(first + 16u * k - 1u), 64);
      if ((j >> 4) >= k) carry += t;
    }
    v += carry;
  }
  return v;
}

// 1 << lg neighbouring lanes of a wavefront (j = 0 .. (1 << lg) - 1) split the staged
// bytes [rs, re) at every delimiter (pat: the delimiter in all four bytes).  Each lane
// takes an equal run of the 16-byte chunks that cover the range and counts its
// delimiters; a prefix sum over the group turns the counts into ordinals, and a second
// walk calls emit(k, position) for the k-th delimiter, k < limit.  Returns the number of
// delimiters in the whole range.  Every lane of a group calls it; those with
// act == false (and, with limit == 0, all of them) emit nothing.
template <class Emit>
__device__ __forceinline__ uint32_t split_bytes(const uint8_t* raw, uint32_t rs, uint32_t re, bool act, uint32_t pat,
                                                uint32_t lg, uint32_t j, uint32_t limit, Emit&& emit) {
  const uint32_t gsz = 1u << lg;
  const uint32_t ab = rs & ~15u;
  const uint32_t nc = (act && re > rs) ? (re - ab + 15u) >> 4 : 0u;  // 16-byte chunks that cover the range
  const uint32_t c = (nc + gsz - 1u) >> lg;                          // chunks per lane
  const uint32_t c0 = min(j * c, nc), c1 = min(c0 + c, nc);
  // one bit per byte of chunk ci: set where the byte is a delimiter (bytes outside the range included)
  auto chunk_bits = [&](uint32_t ci) -> uint32_t {
    const u32x4 w = *reinterpret_cast<const u32x4*>(raw + ab + 16u * ci);
    // flag bytes (0x80 or 0) times weights 1, 2, 4 ...: every sum is 128 times the wanted bits
    uint32_t lo8 = __builtin_amdgcn_udot4(eq_flags(w.x, pat), 0x08040201u, 0u, false);
    lo8 = __builtin_amdgcn_udot4(eq_flags(w.y, pat), 0x80402010u, lo8, false);
    uint32_t hi8 = __builtin_amdgcn_udot4(eq_flags(w.z, pat), 0x08040201u, 0u, false);
    hi8 = __builtin_amdgcn_udot4(eq_flags(w.w, pat), 0x80402010u, hi8, false);
    return (lo8 | (hi8 << 8)) >> 7;
  };
  // the bits [lo, hi) of a mask of n bits that starts at staged position p: those inside the range
  auto inside = [&](uint32_t p, uint32_t n) -> uint64_t {
    const uint32_t lo = rs > p ? rs - p : 0u, hi = min(re - p, n);
    return (hi >= 64u ? ~0ull : (1ull << hi) - 1ull) & (~0ull << lo);
  };
  // A lane with at most four chunks (the usual case) keeps one bit per byte: bit i of (mhi:mlo)
  // is set when byte i of its run is a delimiter.  The second walk then needs no memory at all.
  // With five to eight chunks (long records) two more words (m2, m3) hold the second 64 bytes.
  const bool few = c <= 4u, some = c > 4u && c <= 8u;
  uint32_t mlo = 0, mhi = 0, m2 = 0, m3 = 0, cnt = 0;
  if (few) {
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      if (c0 + q < c1) {
        const uint32_t m16 = chunk_bits(c0 + q);
        if (q == 0) mlo = m16;
        else if (q == 1) mlo |= m16 << 16;
        else if (q == 2) mhi = m16;
        else mhi |= m16 << 16;
      }
    }
    if (c0 < c1) {  // (the lane's run starts before re)
      const uint64_t in = inside(ab + 16u * c0, 64u);
      mlo &= (uint32_t)in;
      mhi &= (uint32_t)(in >> 32);
    }
    cnt = __popc(mlo) + __popc(mhi);
  } else if (some) {
#pragma unroll
    for (uint32_t q = 0; q < 8; ++q) {
      if (c0 + q < c1) {
        const uint32_t m16 = chunk_bits(c0 + q) << (16u * (q & 1u));
        if (q < 2) mlo |= m16;
        else if (q < 4) mhi |= m16;
        else if (q < 6) m2 |= m16;
        else m3 |= m16;
      }
    }
    if (c0 < c1) {
      const uint64_t in = inside(ab + 16u * c0, 64u);
      mlo &= (uint32_t)in;
      mhi &= (uint32_t)(in >> 32);
    }
    if (c0 + 4u < c1) {  // (the second 64 bytes start before re)
      const uint64_t in = inside(ab + 16u * c0 + 64u, 64u);
      m2 &= (uint32_t)in;
      m3 &= (uint32_t)(in >> 32);
    }
    cnt = __popc(mlo) + __popc(mhi) + __popc(m2) + __popc(m3);
  } else {
    for (uint32_t ci = c0; ci < c1; ++ci) cnt += __popc(chunk_bits(ci) & (uint32_t)inside(ab + 16u * ci, 16u));
  }
  const uint32_t incl = group_prefix(cnt, lg, j);
  const uint32_t total = __shfl(incl, (int)(lane_id() | (gsz - 1u)), 64);
  if (!act || !limit) return total;
  uint32_t k = incl - cnt;
  if (few) {
    uint32_t base = ab + 16u * c0;
    uint32_t m = mlo;
    uint32_t room = k < limit ? limit - k : 0u;  // delimiters this lane may still report
#pragma unroll
    for (uint32_t word = 0; word < 2; ++word) {
      uint32_t n = min((uint32_t)__popc(m), room);
      room -= n;
      for (; n; --n) {
        const uint32_t i = (uint32_t)__builtin_ctz(m);  // (m is not zero here)
        emit(k, base + i);
        ++k;
        m &= m - 1u;
      }
      m = mhi;
      base += 32u;
    }
  } else if (some) {
    uint32_t base = ab + 16u * c0;
    uint32_t m = mlo;
    uint32_t room = k < limit ? limit - k : 0u;
#pragma unroll
    for (uint32_t word = 0; word < 4; ++word) {
      uint32_t n = min((uint32_t)__popc(m), room);
      room -= n;
      for (; n; --n) {
        const uint32_t i = (uint32_t)__builtin_ctz(m);  // (m is not zero here)
        emit(k, base + i);
        ++k;
        m &= m - 1u;
      }
      m = word == 0 ? mhi : (word == 1 ? m2 : m3);
      base += 32u;
    }
  } else {
    // second walk of a long run: from delimiter to delimiter.  A window of eight bytes at the
    // current position (any alignment) shows the next one, so every lane places one per turn.
    const uint32_t* raw32 = reinterpret_cast<const uint32_t*>(raw);
    const uint32_t be = min(re, ab + 16u * c1);
    uint32_t p = max(rs, ab + 16u * c0);
    while (p < be) {
      const uint32_t a = p >> 2, sh8 = (p & 3u) * 8u;
      const uint32_t w0 = raw32[a], w1 = raw32[a + 1], w2 = raw32[a + 2];
      const uint32_t f0 = eq_flags(__builtin_amdgcn_alignbit(w1, w0, sh8), pat);
      const uint32_t f1 = eq_flags(__builtin_amdgcn_alignbit(w2, w1, sh8), pat);
      const uint32_t i0 = ((uint32_t)__ffs((int)f0) - 1u) >> 3, i1 = 4u + (((uint32_t)__ffs((int)f1) - 1u) >> 3);
      const uint32_t idx = f0 ? i0 : (f1 ? i1 : 8u);
      p += idx;
      if (idx < 8u && p < be) {
        if (k < limit) emit(k, p);
        ++k;
        ++p;
      }
    }
  }
  return total;
}

}  // namespace
}  // namespace fbx
