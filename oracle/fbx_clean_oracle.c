/*
 * fbx_clean_oracle.c — plain, slow, single-threaded CPU definition of the toy "clean views" stage.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may build, load or call it; it shares no source, header or helper
 * with the HIP library.
 *
 * What it computes.  Section 3 of the paper ("Clean views") names three things that happen to a
 * view before features are extracted from it: null values are filled, fields are extracted from a
 * JSON-like column, and instances are dropped by a custom filter; afterwards every column is
 * non-empty and of a simple type.  The paper gives no algorithm for any of them, so this file
 * writes out the toy contract of this repository, record by record:
 *
 *   - a record is raw[off[i], off[i+1]) without one trailing '\n'; it is cut into exactly F fields
 *     at its tabs (missing fields are empty, fields beyond the F-th are dropped);
 *   - the operators that name a field apply to it in spec order:
 *       fill  field=k value=V   an empty field becomes V
 *       key   field=k name=N    the field is a flat list "k:v;k:v;...": pairs are separated by ';',
 *                               a pair's key ends at its first ':'; the field becomes the value of
 *                               the first pair whose key is exactly N, or empty if there is none
 *                               (a pair without ':' has no value and never matches)
 *       keep  field=k prefix=P  the record is dropped unless the field, as it stands at this point
 *                               of the spec, begins with P
 *   - a record that is kept is written as its F fields joined by '\t' and ended by '\n'; kept
 *     records follow each other in input order; out_off[j] is where the j-th kept record starts
 *     and out_off[n_kept] the length of the output.
 *
 * Parity status.  Pinned by the CPU tests against a Python rendering with bytes.split,
 * bytes.partition and bytes.startswith on hand-built and random records, and by invariants
 * (every output record has exactly F fields; a filled field is never empty; dropping is monotone
 * in the prefix).  There is nothing in the paper to compare values with: parity with the paper's
 * own cleaning operators is unpinned by construction.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

enum { FBXC_OK = 0, FBXC_E_ARG = -1, FBXC_E_SPEC = -2, FBXC_E_NOMEM = -3, FBXC_E_INPUT = -4 };
enum { C_FILL = 1, C_KEY = 2, C_KEEP = 3 };

typedef struct {
  int kind;
  uint32_t field;
  uint8_t arg[256];
  uint32_t arg_len;
} cop_t;

typedef struct {
  uint32_t n_fields;
  cop_t* ops;
  int n_ops;
} cspec_t;

static void set_err(char* err, size_t n, const char* msg, int line) {
  if (err && n) snprintf(err, n, "line %d: %s", line, msg);
}

static int hexval(char c) {
  if (c >= '0' && c <= '9') return c - '0';
  if (c >= 'a' && c <= 'f') return c - 'a' + 10;
  if (c >= 'A' && c <= 'F') return c - 'A' + 10;
  return -1;
}

static int parse_clean_spec(const char* text, size_t len, cspec_t* sp, char* err, size_t errlen) {
  memset(sp, 0, sizeof *sp);
  char* buf = (char*)malloc(len + 1);
  if (!buf) return FBXC_E_NOMEM;
  memcpy(buf, text, len);
  buf[len] = 0;
  int line_no = 0, seen_header = 0, rc = FBXC_OK;
  char* save = NULL;
  for (char* line = strtok_r(buf, "\n", &save); line && rc == FBXC_OK; line = strtok_r(NULL, "\n", &save)) {
    ++line_no;
    char* hash = strchr(line, '#');
    if (hash) *hash = 0;
    char* tok_save = NULL;
    char* word = strtok_r(line, " \t\r", &tok_save);
    if (!word) continue;
    if (!seen_header) {
      char* v = strtok_r(NULL, " \t\r", &tok_save);
      if (strcmp(word, "fbxclean") || !v || strcmp(v, "1")) { set_err(err, errlen, "expected 'fbxclean 1'", line_no); rc = FBXC_E_SPEC; }
      seen_header = 1;
      continue;
    }
    if (!strcmp(word, "fields")) {
      char* v = strtok_r(NULL, " \t\r", &tok_save);
      char* end = NULL;
      unsigned long f = v ? strtoul(v, &end, 10) : 0;
      if (!v || *end || f == 0 || f > 65535 || sp->n_fields) { set_err(err, errlen, "bad or repeated 'fields'", line_no); rc = FBXC_E_SPEC; }
      sp->n_fields = (uint32_t)f;
      continue;
    }
    int kind = !strcmp(word, "fill") ? C_FILL : !strcmp(word, "key") ? C_KEY : !strcmp(word, "keep") ? C_KEEP : 0;
    const char* arg_name = kind == C_FILL ? "value" : kind == C_KEY ? "name" : "prefix";
    if (!kind || !sp->n_fields) { set_err(err, errlen, "unknown operator, or operator before 'fields'", line_no); rc = FBXC_E_SPEC; break; }
    cop_t op;
    memset(&op, 0, sizeof op);
    op.kind = kind;
    int have_field = 0, have_arg = 0;
    for (char* kv = strtok_r(NULL, " \t\r", &tok_save); kv && rc == FBXC_OK; kv = strtok_r(NULL, " \t\r", &tok_save)) {
      char* eq = strchr(kv, '=');
      if (!eq) { set_err(err, errlen, "expected key=value", line_no); rc = FBXC_E_SPEC; break; }
      *eq = 0;
      const char* val = eq + 1;
      if (!strcmp(kv, "field") && !have_field) {
        char* end = NULL;
        unsigned long f = strtoul(val, &end, 10);
        if (!*val || *end || f >= sp->n_fields) { set_err(err, errlen, "field out of range", line_no); rc = FBXC_E_SPEC; }
        op.field = (uint32_t)f;
        have_field = 1;
      } else if (!strcmp(kv, arg_name) && !have_arg) {
        size_t n = strlen(val);
        if (n % 2 || n / 2 > 255) { set_err(err, errlen, "bytes are written as an even number of hex digits, at most 255 bytes", line_no); rc = FBXC_E_SPEC; break; }
        for (size_t i = 0; i < n / 2; ++i) {
          int hi = hexval(val[2 * i]), lo = hexval(val[2 * i + 1]);
          if (hi < 0 || lo < 0) { set_err(err, errlen, "bad hex digit", line_no); rc = FBXC_E_SPEC; break; }
          op.arg[i] = (uint8_t)(hi * 16 + lo);
          if (kind == C_FILL && (op.arg[i] == '\t' || op.arg[i] == '\n')) { set_err(err, errlen, "a fill value holds no tab and no newline", line_no); rc = FBXC_E_SPEC; break; }
        }
        op.arg_len = (uint32_t)(n / 2);
        have_arg = 1;
      } else {
        set_err(err, errlen, "unknown or repeated key", line_no);
        rc = FBXC_E_SPEC;
      }
    }
    if (rc == FBXC_OK && (!have_field || !have_arg)) { set_err(err, errlen, "missing key", line_no); rc = FBXC_E_SPEC; }
    if (rc == FBXC_OK && kind == C_FILL && op.arg_len == 0) { set_err(err, errlen, "a fill value is not empty", line_no); rc = FBXC_E_SPEC; }
    if (rc == FBXC_OK) {
      cop_t* grown = (cop_t*)realloc(sp->ops, (size_t)(sp->n_ops + 1) * sizeof(cop_t));
      if (!grown) { rc = FBXC_E_NOMEM; break; }
      sp->ops = grown;
      sp->ops[sp->n_ops++] = op;
    }
  }
  if (rc == FBXC_OK && (!seen_header || !sp->n_fields)) { set_err(err, errlen, "missing header or 'fields'", line_no); rc = FBXC_E_SPEC; }
  free(buf);
  if (rc != FBXC_OK) { free(sp->ops); sp->ops = NULL; }
  return rc;
}

/* value of the first pair "key:value" (pairs separated by ';') whose key is exactly name */
static void key_lookup(const uint8_t* v, size_t n, const uint8_t* name, size_t name_len, const uint8_t** out, size_t* out_len) {
  size_t p = 0;
  *out = v;
  *out_len = 0;
  for (;;) {
    size_t q = p;
    while (q < n && v[q] != ';') ++q;          /* the pair is v[p, q) */
    size_t c = p;
    while (c < q && v[c] != ':') ++c;          /* its key is v[p, c) if c < q */
    if (c < q && c - p == name_len && memcmp(v + p, name, name_len) == 0) {
      *out = v + c + 1;
      *out_len = q - c - 1;
      return;
    }
    if (q >= n) return;
    p = q + 1;
  }
}

int fbxo_clean(const char* spec, size_t spec_len, const uint8_t* raw, uint64_t raw_len, const uint64_t* off, uint64_t n,
               uint8_t** out_raw, uint64_t* out_len, uint64_t** out_off, uint64_t* n_kept, char* err, size_t errlen) {
  cspec_t sp;
  int rc = parse_clean_spec(spec, spec_len, &sp, err, errlen);
  if (rc != FBXC_OK) return rc;
  for (uint64_t i = 0; i < n; ++i)
    if (off[i] > off[i + 1] || off[i + 1] > raw_len) { free(sp.ops); set_err(err, errlen, "bad record offsets", 0); return FBXC_E_INPUT; }
  size_t cap = 1024, len = 0;
  uint8_t* out = (uint8_t*)malloc(cap);
  uint64_t* offs = (uint64_t*)malloc((size_t)(n + 1) * sizeof(uint64_t));
  const uint8_t** fv = (const uint8_t**)malloc(sp.n_fields * sizeof(uint8_t*));
  size_t* fl = (size_t*)malloc(sp.n_fields * sizeof(size_t));
  uint64_t kept = 0;
  if (!out || !offs || !fv || !fl) rc = FBXC_E_NOMEM;
  for (uint64_t i = 0; i < n && rc == FBXC_OK; ++i) {
    const uint8_t* rec = raw + off[i];
    size_t rn = (size_t)(off[i + 1] - off[i]);
    if (rn && rec[rn - 1] == '\n') --rn;
    size_t p = 0;
    for (uint32_t k = 0; k < sp.n_fields; ++k) {   /* exactly F fields, the missing ones empty */
      size_t q = p;
      while (q < rn && rec[q] != '\t') ++q;
      fv[k] = rec + (p <= rn ? p : rn);
      fl[k] = p <= rn ? q - p : 0;
      p = q < rn ? q + 1 : rn + 1;
    }
    int keep = 1;
    for (int o = 0; o < sp.n_ops && keep; ++o) {
      const cop_t* op = &sp.ops[o];
      const uint32_t k = op->field;
      if (op->kind == C_FILL) {
        if (fl[k] == 0) { fv[k] = op->arg; fl[k] = op->arg_len; }
      } else if (op->kind == C_KEY) {
        key_lookup(fv[k], fl[k], op->arg, op->arg_len, &fv[k], &fl[k]);
      } else {
        keep = fl[k] >= op->arg_len && memcmp(fv[k], op->arg, op->arg_len) == 0;
      }
    }
    if (!keep) continue;
    size_t need = sp.n_fields;                    /* F - 1 tabs and the newline */
    for (uint32_t k = 0; k < sp.n_fields; ++k) need += fl[k];
    if (len + need > cap) {
      while (len + need > cap) cap *= 2;
      uint8_t* grown = (uint8_t*)realloc(out, cap);
      if (!grown) { rc = FBXC_E_NOMEM; break; }
      out = grown;
    }
    offs[kept++] = len;
    for (uint32_t k = 0; k < sp.n_fields; ++k) {
      memcpy(out + len, fv[k], fl[k]);
      len += fl[k];
      out[len++] = k + 1 < sp.n_fields ? '\t' : '\n';
    }
  }
  free(fv);
  free(fl);
  free(sp.ops);
  if (rc != FBXC_OK) { free(out); free(offs); return rc; }
  offs[kept] = len;
  *out_raw = out;
  *out_len = len;
  *out_off = offs;
  *n_kept = kept;
  return FBXC_OK;
}

void fbxo_clean_free(uint8_t* out_raw, uint64_t* out_off) {
  free(out_raw);
  free(out_off);
}
