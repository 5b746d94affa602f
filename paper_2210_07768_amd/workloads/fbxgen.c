/*
 * fbxgen — seeded synthetic ad-log record generator.
 *
 * Produces tab-separated ASCII records whose shapes follow the workloads the
 * feature-extraction path is measured on: single-valued categorical tokens,
 * comma-separated multi-valued lists, decimal numerics and free-text query
 * fields.  It stands in for the proprietary click logs of the paper's
 * evaluation (Section 6, "Models"), which are not available.
 *
 * This file holds no arithmetic of the extraction method itself (no feature
 * hash, no sign mixer, no bucket search): it only draws random text.  Both the
 * CPU oracle's tests and the GPU path's tests feed on its output.
 *
 * Every record is a pure function of (seed, record index), so any record
 * range can be regenerated on its own and in parallel.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { FG_CAT_SINGLE = 0, FG_CAT_MULTI = 1, FG_NUMERIC = 2, FG_TEXT = 3 };

typedef struct {
  int32_t kind;        /* FG_* */
  int32_t len_lo;      /* token (or text) length range, inclusive */
  int32_t len_hi;
  int32_t frac_digits; /* numeric: printed fractional digits, -1 = draw from [0,6] per value */
  double zipf_s;       /* categorical: Zipf exponent (!= 1) */
  double vocab;        /* categorical: vocabulary size V */
  double lambda;       /* multi: list length = 1 + Poisson(lambda) */
  double ln_mu;        /* numeric: x = exp(ln_mu + ln_sigma * N(0,1)) */
  double ln_sigma;
} fbxgen_field;

/* ---- counter-based random numbers (a Murmur3-style finaliser over a Weyl
 * sequence; deliberately not the mixer the extraction method uses) ---------- */
typedef struct { uint64_t s; } rng_t;

static inline uint64_t fin64(uint64_t x) {
  x ^= x >> 33; x *= 0xff51afd7ed558ccdULL;
  x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL;
  x ^= x >> 33;
  return x;
}
static inline rng_t rng_at(uint64_t seed, uint64_t rec, uint64_t field) {
  rng_t r;
  r.s = fin64(seed ^ fin64(rec * 0x9fb21c651e98df25ULL + field + 0x2545f4914f6cdd1dULL));
  return r;
}
static inline uint64_t rng_u64(rng_t* r) {
  r->s += 0xd1342543de82ef95ULL;
  return fin64(r->s);
}
static inline double rng_unit(rng_t* r) { /* [0,1) with 53 bits */
  return (double)(rng_u64(r) >> 11) * (1.0 / 9007199254740992.0);
}

static const char ALNUM[36] = "0123456789abcdefghijklmnopqrstuvwxyz";
static const char TEXTC[40] = "abcdefghijklmnopqrstuvwxyz0123456789  -.";

/* Zipf(s) rank in [1, V] by inverting the continuous approximation of the CDF. */
static inline uint64_t zipf_rank(rng_t* r, double s, double V) {
  double u = rng_unit(r);
  double e = 1.0 - s;
  double x = pow((pow(V + 1.0, e) - 1.0) * u + 1.0, 1.0 / e);
  if (!(x >= 1.0)) x = 1.0;
  if (x > V) x = V;
  return (uint64_t)x;
}

/* The token of a vocabulary rank: length and bytes depend on the rank only. */
static inline size_t put_token(uint8_t* out, uint64_t rank, int lo, int hi) {
  uint64_t h = fin64(rank * 0x9e3779b97f4a7c15ULL + 0x7f4a7c15ULL);
  int len = lo + (int)(h % (uint64_t)(hi - lo + 1));
  uint64_t x = 0;
  int have = 0;
  for (int i = 0; i < len; ++i) {
    if (have == 0) { h = fin64(h + 0x632be59bd9b4e019ULL); x = h; have = 12; }
    out[i] = (uint8_t)ALNUM[x % 36];
    x /= 36; --have;
  }
  return (size_t)len;
}

static inline int poisson(rng_t* r, double lambda) {
  double u = rng_unit(r), p = exp(-lambda), c = p;
  int k = 0;
  while (u > c && k < 200) { ++k; p *= lambda / k; c += p; }
  return k;
}

static inline size_t put_u64_dec(uint8_t* out, uint64_t v) {
  char tmp[24]; int n = 0;
  do { tmp[n++] = (char)('0' + v % 10); v /= 10; } while (v);
  for (int i = 0; i < n; ++i) out[i] = (uint8_t)tmp[n - 1 - i];
  return (size_t)n;
}

static inline size_t put_numeric(uint8_t* out, rng_t* r, const fbxgen_field* f) {
  double u1 = rng_unit(r), u2 = rng_unit(r);
  double z = sqrt(-2.0 * log(1.0 - u1)) * cos(6.283185307179586 * u2);
  double x = exp(f->ln_mu + f->ln_sigma * z);
  if (!(x < 9.0e12)) x = 9.0e12;
  uint64_t micro = (uint64_t)(x * 1.0e6);
  int k = f->frac_digits;
  if (k < 0) k = (int)(rng_u64(r) % 7);
  size_t n = put_u64_dec(out, micro / 1000000ULL);
  if (k > 0) {
    uint64_t frac = micro % 1000000ULL;
    char d[6];
    for (int i = 5; i >= 0; --i) { d[i] = (char)('0' + frac % 10); frac /= 10; }
    out[n++] = '.';
    for (int i = 0; i < k; ++i) out[n++] = (uint8_t)d[i];
  }
  return n;
}

/* Upper bound on the bytes one record can take (used to size scratch). */
static size_t record_bound(const fbxgen_field* fields, int F) {
  size_t b = 2;
  for (int k = 0; k < F; ++k) {
    const fbxgen_field* f = &fields[k];
    size_t hi = (size_t)(f->len_hi > 0 ? f->len_hi : 1);
    switch (f->kind) {
      case FG_CAT_SINGLE: b += hi + 1; break;
      case FG_CAT_MULTI:  b += 202 * (hi + 1); break;
      case FG_NUMERIC:    b += 32; break;
      default:            b += hi + 1; break;
    }
  }
  return b;
}

static size_t make_record(uint8_t* out, uint64_t seed, uint64_t rec,
                          const fbxgen_field* fields, int F) {
  size_t n = 0;
  for (int k = 0; k < F; ++k) {
    const fbxgen_field* f = &fields[k];
    rng_t r = rng_at(seed, rec, (uint64_t)k);
    if (k) out[n++] = '\t';
    switch (f->kind) {
      case FG_CAT_SINGLE:
        n += put_token(out + n, zipf_rank(&r, f->zipf_s, f->vocab), f->len_lo, f->len_hi);
        break;
      case FG_CAT_MULTI: {
        int items = 1 + poisson(&r, f->lambda);
        for (int i = 0; i < items; ++i) {
          if (i) out[n++] = ',';
          n += put_token(out + n, zipf_rank(&r, f->zipf_s, f->vocab), f->len_lo, f->len_hi);
        }
        break;
      }
      case FG_NUMERIC:
        n += put_numeric(out + n, &r, f);
        break;
      default: {
        int len = f->len_lo + (int)(rng_u64(&r) % (uint64_t)(f->len_hi - f->len_lo + 1));
        uint64_t x = 0; int have = 0;
        for (int i = 0; i < len; ++i) {
          if (have == 0) { x = rng_u64(&r); have = 12; }
          out[n++] = (uint8_t)TEXTC[x % 40];
          x /= 40; --have;
        }
        break;
      }
    }
  }
  out[n++] = '\n';
  return n;
}

/*
 * Generate records [rec_begin, rec_begin + n_records).
 *   out      : byte buffer of capacity out_cap (may be NULL with out_cap 0 to
 *              query the size only)
 *   rec_off  : n_records + 1 offsets relative to out (always filled)
 * Returns the total number of bytes the records take; nothing is written to
 * `out` unless the total fits in out_cap.
 */
uint64_t fbxgen_generate(uint64_t seed, const fbxgen_field* fields, int32_t F,
                         uint64_t rec_begin, uint64_t n_records,
                         uint8_t* out, uint64_t out_cap, uint64_t* rec_off) {
  const size_t bound = record_bound(fields, F);
  const uint64_t CH = 2048; /* records per work item */
  const uint64_t n_chunks = (n_records + CH - 1) / CH;
  uint8_t** bufs = (uint8_t**)calloc(n_chunks ? n_chunks : 1, sizeof(uint8_t*));
  uint64_t* lens = (uint64_t*)calloc(n_records ? n_records : 1, sizeof(uint64_t));
  if (!bufs || !lens) { free(bufs); free(lens); return 0; }

#pragma omp parallel
  {
    uint8_t* scratch = (uint8_t*)malloc(bound);
#pragma omp for schedule(dynamic, 1)
    for (int64_t c = 0; c < (int64_t)n_chunks; ++c) {
      uint64_t r0 = (uint64_t)c * CH, r1 = r0 + CH < n_records ? r0 + CH : n_records;
      size_t cap = 1 << 16, used = 0;
      uint8_t* b = (uint8_t*)malloc(cap);
      for (uint64_t r = r0; r < r1; ++r) {
        size_t n = make_record(scratch, seed, rec_begin + r, fields, F);
        if (used + n > cap) { while (used + n > cap) cap *= 2; b = (uint8_t*)realloc(b, cap); }
        memcpy(b + used, scratch, n);
        used += n; lens[r] = n;
      }
      bufs[c] = b;
    }
    free(scratch);
  }

  uint64_t total = 0;
  for (uint64_t r = 0; r < n_records; ++r) { rec_off[r] = total; total += lens[r]; }
  rec_off[n_records] = total;

  if (out && total <= out_cap) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t c = 0; c < (int64_t)n_chunks; ++c) {
      uint64_t r0 = (uint64_t)c * CH, r1 = r0 + CH < n_records ? r0 + CH : n_records;
      memcpy(out + rec_off[r0], bufs[c], rec_off[r1] - rec_off[r0]);
    }
  }
  for (uint64_t c = 0; c < n_chunks; ++c) free(bufs[c]);
  free(bufs); free(lens);
  return total;
}
