/*
 * fbx_oracle.c — plain, slow, single-threaded CPU definition of the batched
 * feature-extraction path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may build, load or call it.  It
 * shares no source, header, table or helper with the HIP library; the two
 * meet only in the test harness that compares their outputs.
 *
 * What it computes.  The paper (Section 3, "Extract features") describes the
 * stage as a collection of per-feature operators evaluated on the rows of one
 * structured table, with dependencies between operators resolved beforehand
 * (Section 4, "Scheduling"); the only operator it spells out is splitting a
 * string at a delimiter (Section 5, first paragraph), and "feature
 * combinations" are named in Section 1.  The paper defines no hash, no
 * combination rule, no bucketing rule and no output layout, so every operator
 * below follows the written contract of this repository (the readings are
 * listed where each function is defined).  Because that contract is an exact
 * definition, not an approximation, this file simply writes the definition
 * out: record by record, operator by operator in spec order, one growable
 * list of 64-bit signs per operator.
 *
 * Parity status.  All arithmetic here is pinned by the CPU tests against
 * published FNV-1a-64 and SplitMix64 values, Python library routines
 * (bytes.split, bisect, Decimal, startswith), hand-built records and count
 * invariants.  Parity with sign values of the paper's own system is unpinned
 * by construction: the paper prints none.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ status */
enum { FBXO_OK = 0, FBXO_E_ARG = -1, FBXO_E_SPEC = -2, FBXO_E_NOMEM = -3, FBXO_E_INPUT = -4 };

enum { K_HASH = 1, K_NGRAM = 2, K_BUCKET = 3, K_FILTER = 4, K_CROSS = 5, K_CONCAT = 6 };

typedef struct {
  char id[64];
  int kind;
  uint32_t slot;
  uint64_t seed;
  int emit;
  uint32_t field;
  int multi;
  int n;                 /* n-gram width */
  int64_t* bounds;       /* bucket boundaries, non-decreasing */
  uint32_t n_bounds;
  uint8_t prefix[256];
  uint32_t prefix_len;
  int a, b;              /* input operator indices (cross / concat) */
  int layer;             /* 1 = reads raw fields only */
  uint32_t fixed_arity;  /* >0: always exactly this many signs per record */
} op_t;

typedef struct {
  uint32_t n_fields;
  op_t* ops;
  int n_ops;
  int n_layers;
} spec_t;

typedef struct { uint64_t* v; size_t n, cap; } list_t;

typedef struct {
  uint32_t slot_id;
  uint32_t fixed_arity;
  uint64_t n_values;
  uint64_t* values;
  uint64_t* offsets; /* always explicit: n_records + 1 entries */
} fbxo_slot;

typedef struct {
  uint64_t n_records;
  uint64_t n_values_total;
  uint64_t n_malformed_numeric;
  uint32_t n_slots;
  uint32_t n_layers;
  fbxo_slot* slots;
} fbxo_result;

/* ------------------------------------------------------- scalar arithmetic */

/*
 * Slot-seeded string hash (contract point "string hash"): the 64-bit FNV-1a
 * hash of the message formed by the seed's eight little-endian bytes followed
 * by the token bytes.  FNV-1a: start from the offset basis; for every byte,
 * xor it in, then multiply by the FNV prime modulo 2^64.
 */
uint64_t fbxo_hash_bytes(uint64_t seed, const uint8_t* m, size_t n) {
  uint64_t h = 0xcbf29ce484222325ULL;
  for (int i = 0; i < 8; ++i) {
    h ^= (uint8_t)(seed >> (8 * i));
    h *= 0x100000001b3ULL;
  }
  for (size_t i = 0; i < n; ++i) {
    h ^= m[i];
    h *= 0x100000001b3ULL;
  }
  return h;
}

/* Fixed-width mixer (contract point "mixer"): the SplitMix64 output function. */
uint64_t fbxo_mix64(uint64_t x) {
  x ^= x >> 30;
  x *= 0xbf58476d1ce4e5b9ULL;
  x ^= x >> 27;
  x *= 0x94d049bb133111ebULL;
  x ^= x >> 31;
  return x;
}

/*
 * Cross of two signs under a slot key K = mix64(seed) (contract point "cross
 * combination"): mix64(mix64(a + K) + b), additions modulo 2^64.  Not
 * commutative in (a, b).
 */
uint64_t fbxo_cross(uint64_t K, uint64_t a, uint64_t b) {
  return fbxo_mix64(fbxo_mix64(a + K) + b);
}

/*
 * Decimal text to signed micro-units (contract point "numeric grammar"):
 * optional '-', integer digits, optional '.' and fractional digits; the scan
 * stops at the first byte that fits none of these.  Only the first six
 * fractional digits count (truncation toward zero).  Accumulation is modulo
 * 2^64 and the sign is applied last, so overflow is defined.  *malformed is
 * set when the scan stopped before the end of the token or met no digit.
 */
int64_t fbxo_parse_micro(const uint8_t* t, size_t n, int* malformed) {
  size_t i = 0;
  int neg = 0, digits = 0, nfrac = 0;
  uint64_t ip = 0, fp = 0;
  if (i < n && t[i] == '-') { neg = 1; ++i; }
  while (i < n && t[i] >= '0' && t[i] <= '9') { ip = ip * 10u + (uint64_t)(t[i] - '0'); ++digits; ++i; }
  if (i < n && t[i] == '.') {
    ++i;
    while (i < n && t[i] >= '0' && t[i] <= '9') {
      if (nfrac < 6) { fp = fp * 10u + (uint64_t)(t[i] - '0'); ++nfrac; }
      ++digits; ++i;
    }
  }
  while (nfrac < 6) { fp *= 10u; ++nfrac; }
  uint64_t v = ip * 1000000u + fp;
  if (neg) v = (uint64_t)0 - v;
  if (malformed) *malformed = (i < n) || digits == 0;
  return (int64_t)v;
}

/* Bucket index (contract point "bucketise"): how many boundaries are <= v. */
uint32_t fbxo_bucket_index(const int64_t* bounds, uint32_t n, int64_t v) {
  uint32_t c = 0;
  for (uint32_t j = 0; j < n; ++j)
    if (bounds[j] <= v) ++c;
  return c;
}

/* ------------------------------------------------------------ spec parsing */
static void set_err(char* err, size_t errlen, const char* fmt, int line, const char* what) {
  if (err && errlen) snprintf(err, errlen, fmt, line, what);
}

static int parse_u64(const char* s, uint64_t* out) {
  if (!*s) return 0;
  uint64_t v = 0;
  for (; *s; ++s) {
    if (*s < '0' || *s > '9') return 0;
    uint64_t d = (uint64_t)(*s - '0');
    if (v > (UINT64_MAX - d) / 10u) return 0;
    v = v * 10u + d;
  }
  *out = v;
  return 1;
}

static int parse_i64(const char* s, int64_t* out) {
  int neg = 0;
  if (*s == '-') { neg = 1; ++s; }
  uint64_t v;
  if (!parse_u64(s, &v)) return 0;
  if (neg) { if (v > (uint64_t)INT64_MAX + 1u) return 0; *out = (int64_t)((uint64_t)0 - v); }
  else { if (v > (uint64_t)INT64_MAX) return 0; *out = (int64_t)v; }
  return 1;
}

static int id_ok(const char* s) {
  size_t n = strlen(s);
  if (n == 0 || n > 63) return 0;
  for (size_t i = 0; i < n; ++i) {
    char c = s[i];
    if (!((c >= '0' && c <= '9') || (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_')) return 0;
  }
  return 1;
}

static int find_op(const spec_t* sp, const char* id) {
  for (int i = 0; i < sp->n_ops; ++i)
    if (strcmp(sp->ops[i].id, id) == 0) return i;
  return -1;
}

static int hexval(char c) {
  if (c >= '0' && c <= '9') return c - '0';
  if (c >= 'a' && c <= 'f') return c - 'a' + 10;
  if (c >= 'A' && c <= 'F') return c - 'A' + 10;
  return -1;
}

static void spec_free(spec_t* sp) {
  for (int i = 0; i < sp->n_ops; ++i) free(sp->ops[i].bounds);
  free(sp->ops);
  sp->ops = NULL; sp->n_ops = 0;
}

/* Key bits, to check that each operator kind gets exactly its own keys. */
enum { KB_SLOT = 1, KB_SEED = 2, KB_EMIT = 4, KB_FIELD = 8, KB_MULTI = 16, KB_N = 32, KB_BOUNDS = 64,
       KB_PREFIX = 128, KB_A = 256, KB_B = 512 };

static int parse_spec(const char* text, size_t len, spec_t* sp, char* err, size_t errlen) {
  memset(sp, 0, sizeof(*sp));
  char* buf = (char*)malloc(len + 1);
  if (!buf) return FBXO_E_NOMEM;
  memcpy(buf, text, len);
  buf[len] = 0;
  for (size_t i = 0; i < len; ++i)
    if (buf[i] == 0) { free(buf); set_err(err, errlen, "line %d: %s", 0, "NUL byte in spec"); return FBXO_E_SPEC; }
  int cap = 0, lineno = 0, stage = 0, rc = FBXO_OK;
  char* save = NULL;
  char* p = buf;
  while (p && *p) {
    char* nl = strchr(p, '\n');
    if (nl) *nl = 0;
    char* line = p;
    p = nl ? nl + 1 : NULL;
    ++lineno;
    while (*line == ' ' || *line == '\r') ++line;
    size_t L = strlen(line);
    while (L && (line[L - 1] == ' ' || line[L - 1] == '\r')) line[--L] = 0;
    if (L == 0 || line[0] == '#') continue;
#define FAIL(msg) do { set_err(err, errlen, "line %d: %s", lineno, msg); rc = FBXO_E_SPEC; goto done; } while (0)
    char* tok = strtok_r(line, " ", &save);
    if (stage == 0) {
      char* ver = strtok_r(NULL, " ", &save);
      if (strcmp(tok, "fbx") != 0 || !ver || strcmp(ver, "1") != 0 || strtok_r(NULL, " ", &save)) FAIL("expected 'fbx 1'");
      stage = 1;
      continue;
    }
    if (stage == 1) {
      char* nf = strtok_r(NULL, " ", &save);
      uint64_t F;
      if (strcmp(tok, "fields") != 0 || !nf || !parse_u64(nf, &F) || F < 1 || F > 65535 || strtok_r(NULL, " ", &save))
        FAIL("expected 'fields <1..65535>'");
      sp->n_fields = (uint32_t)F;
      stage = 2;
      continue;
    }
    if (strcmp(tok, "op") != 0) FAIL("expected 'op'");
    char* id = strtok_r(NULL, " ", &save);
    char* kind = strtok_r(NULL, " ", &save);
    if (!id || !kind || !id_ok(id)) FAIL("bad operator id");
    if (find_op(sp, id) >= 0) FAIL("duplicate operator id");
    if (sp->n_ops >= 65535) FAIL("too many operators");
    if (sp->n_ops == cap) {
      cap = cap ? cap * 2 : 64;
      op_t* no = (op_t*)realloc(sp->ops, (size_t)cap * sizeof(op_t));
      if (!no) { rc = FBXO_E_NOMEM; goto done; }
      sp->ops = no;
    }
    op_t* o = &sp->ops[sp->n_ops];
    memset(o, 0, sizeof(*o));
    strcpy(o->id, id);
    o->a = o->b = -1;
    int need;
    if (!strcmp(kind, "hash")) { o->kind = K_HASH; need = KB_SLOT | KB_SEED | KB_EMIT | KB_FIELD | KB_MULTI; }
    else if (!strcmp(kind, "ngram")) { o->kind = K_NGRAM; need = KB_SLOT | KB_SEED | KB_EMIT | KB_FIELD | KB_N; }
    else if (!strcmp(kind, "bucket")) { o->kind = K_BUCKET; need = KB_SLOT | KB_SEED | KB_EMIT | KB_FIELD | KB_MULTI | KB_BOUNDS; }
    else if (!strcmp(kind, "filter")) { o->kind = K_FILTER; need = KB_SLOT | KB_SEED | KB_EMIT | KB_FIELD | KB_MULTI | KB_PREFIX; }
    else if (!strcmp(kind, "cross")) { o->kind = K_CROSS; need = KB_SLOT | KB_SEED | KB_EMIT | KB_A | KB_B; }
    else if (!strcmp(kind, "concat")) { o->kind = K_CONCAT; need = KB_SLOT | KB_EMIT | KB_A | KB_B; }
    else FAIL("unknown operator kind");
    int seen = 0;
    for (char* kv = strtok_r(NULL, " ", &save); kv; kv = strtok_r(NULL, " ", &save)) {
      char* eq = strchr(kv, '=');
      if (!eq) { free(o->bounds); o->bounds = NULL; FAIL("expected key=value"); }
      *eq = 0;
      const char* key = kv;
      const char* val = eq + 1;
      int bit = 0;
      uint64_t u = 0;
      int bad = 0;
      if (!strcmp(key, "slot")) { bit = KB_SLOT; if (!parse_u64(val, &u) || u > 0xffffffffu) bad = 1; o->slot = (uint32_t)u; }
      else if (!strcmp(key, "seed")) { bit = KB_SEED; if (!parse_u64(val, &u)) bad = 1; o->seed = u; }
      else if (!strcmp(key, "emit")) { bit = KB_EMIT; if (!parse_u64(val, &u) || u > 1) bad = 1; o->emit = (int)u; }
      else if (!strcmp(key, "field")) { bit = KB_FIELD; if (!parse_u64(val, &u) || u >= sp->n_fields) bad = 1; o->field = (uint32_t)u; }
      else if (!strcmp(key, "multi")) { bit = KB_MULTI; if (!parse_u64(val, &u) || u > 1) bad = 1; o->multi = (int)u; }
      else if (!strcmp(key, "n")) { bit = KB_N; if (!parse_u64(val, &u) || u < 1 || u > 8) bad = 1; o->n = (int)u; }
      else if (!strcmp(key, "a") || !strcmp(key, "b")) {
        bit = key[0] == 'a' ? KB_A : KB_B;
        int ref = find_op(sp, val); /* only earlier lines are visible: no forward or self reference */
        if (ref < 0) bad = 1;
        if (key[0] == 'a') o->a = ref; else o->b = ref;
      } else if (!strcmp(key, "bounds")) {
        bit = KB_BOUNDS;
        if (seen & KB_BOUNDS) bad = 1;
        size_t vl = strlen(val), cnt = vl ? 1 : 0;
        for (size_t i = 0; i < vl; ++i) if (val[i] == ',') ++cnt;
        if (cnt > 4096) bad = 1;
        if (!bad && cnt) {
          o->bounds = (int64_t*)malloc(cnt * sizeof(int64_t));
          char* dup = strdup(val);
          uint32_t k = 0;
          /* strtok_r would skip empty items, so walk the commas by hand */
          char* cur = dup;
          while (cur) {
            char* c = strchr(cur, ',');
            if (c) *c = 0;
            int64_t b;
            if (!parse_i64(cur, &b)) { bad = 1; break; }
            if (k && b < o->bounds[k - 1]) { bad = 1; break; }
            o->bounds[k++] = b;
            cur = c ? c + 1 : NULL;
          }
          free(dup);
          o->n_bounds = k;
        }
      } else if (!strcmp(key, "prefix")) {
        bit = KB_PREFIX;
        size_t vl = strlen(val);
        if (vl % 2 || vl / 2 > 255) bad = 1;
        for (size_t i = 0; !bad && i < vl; i += 2) {
          int hi = hexval(val[i]), lo = hexval(val[i + 1]);
          if (hi < 0 || lo < 0) bad = 1; else o->prefix[i / 2] = (uint8_t)(hi * 16 + lo);
        }
        o->prefix_len = (uint32_t)(vl / 2);
      } else { free(o->bounds); o->bounds = NULL; FAIL("unknown key"); }
      if (bad || (seen & bit) || !(need & bit)) { free(o->bounds); o->bounds = NULL; FAIL("bad, repeated or misplaced key"); }
      seen |= bit;
    }
    if (seen != need) { free(o->bounds); o->bounds = NULL; FAIL("missing key"); }
    /* Layer rule (Section 4, "Scheduling"): operators without dependencies
     * form the first layer, the others sit one below their deepest input. */
    if (o->kind == K_CROSS || o->kind == K_CONCAT) {
      int la = sp->ops[o->a].layer, lb = sp->ops[o->b].layer;
      o->layer = 1 + (la > lb ? la : lb);
      uint32_t fa = sp->ops[o->a].fixed_arity, fb = sp->ops[o->b].fixed_arity;
      if (fa && fb) {
        uint64_t k = o->kind == K_CROSS ? (uint64_t)fa * fb : (uint64_t)fa + fb;
        o->fixed_arity = k <= 0xffffffffu ? (uint32_t)k : 0;
      }
    } else {
      o->layer = 1;
      o->fixed_arity = ((o->kind == K_HASH || o->kind == K_BUCKET) && !o->multi) ? 1 : 0;
    }
    if (o->layer > sp->n_layers) sp->n_layers = o->layer;
    if (o->emit)
      for (int i = 0; i < sp->n_ops; ++i)
        if (sp->ops[i].emit && sp->ops[i].slot == o->slot) { free(o->bounds); o->bounds = NULL; FAIL("duplicate emitted slot"); }
    sp->n_ops++;
  }
  if (stage < 2) { set_err(err, errlen, "line %d: %s", lineno, "spec needs 'fbx 1' and 'fields'"); rc = FBXO_E_SPEC; }
done:
  free(buf);
  if (rc != FBXO_OK) spec_free(sp);
  return rc;
#undef FAIL
}

/* ------------------------------------------------------------- list helper */
static int push(list_t* l, uint64_t x) {
  if (l->n == l->cap) {
    size_t nc = l->cap ? l->cap * 2 : 16;
    uint64_t* nv = (uint64_t*)realloc(l->v, nc * sizeof(uint64_t));
    if (!nv) return 0;
    l->v = nv; l->cap = nc;
  }
  l->v[l->n++] = x;
  return 1;
}

/* ------------------------------------------------------ one record, one op */

/* Field k of a record (contract point "field framing"): the bytes between the
 * k-th and (k+1)-th tab; a record with too few tabs has empty trailing fields. */
static void field_span(const uint8_t* rec, size_t n, uint32_t k, size_t* s, size_t* e) {
  size_t pos = 0;
  for (uint32_t f = 0; f < k; ++f) {
    while (pos < n && rec[pos] != '\t') ++pos;
    if (pos == n) { *s = *e = n; return; }
    ++pos; /* step over the tab */
  }
  size_t end = pos;
  while (end < n && rec[end] != '\t') ++end;
  *s = pos; *e = end;
}

static int token_sign(const op_t* o, const uint8_t* t, size_t n, list_t* out, uint64_t* malformed) {
  switch (o->kind) {
    case K_HASH:
      return push(out, fbxo_hash_bytes(o->seed, t, n));
    case K_FILTER:
      if (n >= o->prefix_len && memcmp(t, o->prefix, o->prefix_len) == 0)
        return push(out, fbxo_hash_bytes(o->seed, t, n));
      return 1;
    case K_BUCKET: {
      int bad = 0;
      int64_t v = fbxo_parse_micro(t, n, &bad);
      if (bad) ++*malformed;
      uint32_t idx = fbxo_bucket_index(o->bounds, o->n_bounds, v);
      return push(out, fbxo_mix64(fbxo_mix64(o->seed) + (uint64_t)idx));
    }
    default:
      return 0;
  }
}

static int eval_op(const spec_t* sp, int oi, const uint8_t* rec, size_t n, list_t* lists, uint64_t* malformed) {
  const op_t* o = &sp->ops[oi];
  list_t* out = &lists[oi];
  out->n = 0;
  if (o->kind == K_CROSS) {
    const list_t* A = &lists[o->a];
    const list_t* B = &lists[o->b];
    uint64_t K = fbxo_mix64(o->seed);
    for (size_t i = 0; i < A->n; ++i)
      for (size_t j = 0; j < B->n; ++j)
        if (!push(out, fbxo_cross(K, A->v[i], B->v[j]))) return 0;
    return 1;
  }
  if (o->kind == K_CONCAT) {
    /* a and b may name the same operator, and may alias nothing else: copy by index */
    size_t na = lists[o->a].n, nb = lists[o->b].n;
    for (size_t i = 0; i < na; ++i) if (!push(out, lists[o->a].v[i])) return 0;
    for (size_t j = 0; j < nb; ++j) if (!push(out, lists[o->b].v[j])) return 0;
    return 1;
  }
  size_t s, e;
  field_span(rec, n, o->field, &s, &e);
  if (o->kind == K_NGRAM) {
    size_t L = e - s, g = (size_t)o->n;
    for (size_t k = 0; k + g <= L; ++k)
      if (!push(out, fbxo_hash_bytes(o->seed, rec + s + k, g))) return 0;
    return 1;
  }
  if (!o->multi) return token_sign(o, rec + s, e - s, out, malformed);
  /* multi-valued: split at every comma; empty items are kept (bytes.split semantics) */
  size_t t0 = s;
  for (size_t i = s; i <= e; ++i) {
    if (i == e || rec[i] == ',') {
      if (!token_sign(o, rec + t0, i - t0, out, malformed)) return 0;
      t0 = i + 1;
    }
  }
  return 1;
}

/* ----------------------------------------------------------------- extract */
void fbxo_free(fbxo_result* r) {
  if (!r || !r->slots) return;
  for (uint32_t i = 0; i < r->n_slots; ++i) { free(r->slots[i].values); free(r->slots[i].offsets); }
  free(r->slots);
  memset(r, 0, sizeof(*r));
}

int fbxo_extract(const char* spec, size_t spec_len, const uint8_t* raw, uint64_t raw_len,
                 const uint64_t* rec_off, uint64_t n_records, fbxo_result* out, char* err, size_t errlen) {
  if (!spec || !out || (!rec_off && n_records) || (!raw && raw_len)) return FBXO_E_ARG;
  memset(out, 0, sizeof(*out));
  spec_t sp;
  int rc = parse_spec(spec, spec_len, &sp, err, errlen);
  if (rc != FBXO_OK) return rc;
  /* record framing: offsets non-decreasing and inside the buffer */
  for (uint64_t r = 0; r < n_records; ++r)
    if (rec_off[r] > rec_off[r + 1] || rec_off[r + 1] > raw_len) {
      set_err(err, errlen, "record %d: %s", (int)r, "offsets must be non-decreasing and within raw_len");
      spec_free(&sp);
      return FBXO_E_INPUT;
    }
  uint32_t n_slots = 0;
  for (int i = 0; i < sp.n_ops; ++i) n_slots += (uint32_t)sp.ops[i].emit;
  list_t* lists = (list_t*)calloc((size_t)(sp.n_ops ? sp.n_ops : 1), sizeof(list_t));
  list_t* outs = (list_t*)calloc(n_slots ? n_slots : 1, sizeof(list_t));
  out->slots = (fbxo_slot*)calloc(n_slots ? n_slots : 1, sizeof(fbxo_slot));
  int* slot_of_op = (int*)malloc((size_t)(sp.n_ops ? sp.n_ops : 1) * sizeof(int));
  int ok = lists && outs && out->slots && slot_of_op;
  out->n_slots = n_slots;
  out->n_records = n_records;
  out->n_layers = (uint32_t)sp.n_layers;
  if (ok) {
    uint32_t s = 0;
    for (int i = 0; i < sp.n_ops; ++i) {
      slot_of_op[i] = -1;
      if (!sp.ops[i].emit) continue;
      slot_of_op[i] = (int)s;
      out->slots[s].slot_id = sp.ops[i].slot;
      out->slots[s].fixed_arity = sp.ops[i].fixed_arity;
      out->slots[s].offsets = (uint64_t*)calloc(n_records + 1, sizeof(uint64_t));
      if (!out->slots[s].offsets) ok = 0;
      ++s;
    }
  }
  for (uint64_t r = 0; ok && r < n_records; ++r) {
    const uint8_t* rec = raw + rec_off[r];
    size_t n = (size_t)(rec_off[r + 1] - rec_off[r]);
    if (n && rec[n - 1] == '\n') --n; /* one trailing newline is not part of the record */
    for (int i = 0; ok && i < sp.n_ops; ++i) {
      if (!eval_op(&sp, i, rec, n, lists, &out->n_malformed_numeric)) { ok = 0; break; }
      int s = slot_of_op[i];
      if (s < 0) continue;
      for (size_t k = 0; k < lists[i].n; ++k)
        if (!push(&outs[s], lists[i].v[k])) { ok = 0; break; }
      out->slots[s].offsets[r + 1] = outs[s].n;
    }
  }
  for (uint32_t s = 0; s < n_slots; ++s) {
    out->slots[s].values = outs[s].v;
    out->slots[s].n_values = outs[s].n;
    out->n_values_total += outs[s].n;
  }
  for (int i = 0; i < sp.n_ops; ++i) free(lists[i].v);
  free(lists); free(outs); free(slot_of_op);
  spec_free(&sp);
  if (!ok) { fbxo_free(out); return FBXO_E_NOMEM; }
  return FBXO_OK;
}

/*
 * Layer of every operator, in spec order (1-based), for checking the layer
 * partition on its own.  Returns the operator count, or a negative status.
 */
int fbxo_spec_layers(const char* spec, size_t spec_len, int32_t* layer_out, int32_t cap,
                     uint32_t* arity_out, char* err, size_t errlen) {
  spec_t sp;
  int rc = parse_spec(spec, spec_len, &sp, err, errlen);
  if (rc != FBXO_OK) return rc;
  int n = sp.n_ops;
  for (int i = 0; i < n && i < cap; ++i) {
    if (layer_out) layer_out[i] = sp.ops[i].layer;
    if (arity_out) arity_out[i] = sp.ops[i].fixed_arity;
  }
  spec_free(&sp);
  return n;
}
