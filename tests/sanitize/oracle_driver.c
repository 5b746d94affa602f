/* Runs the CPU oracles on spec and record files given on the command line, for a build with
 * -fsanitize=address,undefined (test infrastructure: see tests/test_host_sanitizers.py).
 * usage: oracle_driver extract|clean <spec file> <raw file> <offsets file (u64, n + 1 entries)> */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint32_t slot_id, fixed_arity; uint64_t n_values; uint64_t* values; uint64_t* offsets; } slot_t;
typedef struct { uint64_t n_records, n_values_total, n_malformed_numeric; uint32_t n_slots, n_layers; slot_t* slots; } result_t;
int fbxo_extract(const char*, size_t, const uint8_t*, uint64_t, const uint64_t*, uint64_t, result_t*, char*, size_t);
void fbxo_free(result_t*);
int fbxo_spec_layers(const char*, size_t, int32_t*, int32_t, uint32_t*, char*, size_t);
int fbxo_clean(const char*, size_t, const uint8_t*, uint64_t, const uint64_t*, uint64_t, uint8_t**, uint64_t*, uint64_t**, uint64_t*,
               char*, size_t);
void fbxo_clean_free(uint8_t*, uint64_t*);

static uint8_t* slurp(const char* path, size_t* n) {
  FILE* f = fopen(path, "rb");
  if (!f) { perror(path); exit(2); }
  fseek(f, 0, SEEK_END);
  long len = ftell(f);
  fseek(f, 0, SEEK_SET);
  uint8_t* buf = (uint8_t*)malloc((size_t)len + 1);
  if (len && fread(buf, 1, (size_t)len, f) != (size_t)len) { perror("read"); exit(2); }
  fclose(f);
  *n = (size_t)len;
  return buf;
}

int main(int argc, char** argv) {
  if (argc != 5) { fprintf(stderr, "usage: %s extract|clean spec raw offsets\n", argv[0]); return 2; }
  size_t spec_len, raw_len, off_len;
  uint8_t* spec = slurp(argv[2], &spec_len);
  uint8_t* raw = slurp(argv[3], &raw_len);
  uint8_t* off_bytes = slurp(argv[4], &off_len);
  uint64_t* off = (uint64_t*)malloc(off_len + 8);   /* (an exact-size, aligned copy: overruns are seen) */
  memcpy(off, off_bytes, off_len);
  const uint64_t n = off_len >= 8 ? off_len / 8 - 1 : 0;
  char err[256] = "";
  int rc;
  if (!strcmp(argv[1], "extract")) {
    int32_t n_ops = fbxo_spec_layers((const char*)spec, spec_len, NULL, 0, NULL, err, sizeof err);
    if (n_ops > 0) {
      int32_t* layers = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_ops);
      uint32_t* arity = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)n_ops);
      fbxo_spec_layers((const char*)spec, spec_len, layers, n_ops, arity, err, sizeof err);
      free(layers);
      free(arity);
    }
    result_t res;
    memset(&res, 0, sizeof res);
    rc = fbxo_extract((const char*)spec, spec_len, raw_len ? raw : NULL, raw_len, off, n, &res, err, sizeof err);
    if (rc == 0) {
      uint64_t sum = 0;
      for (uint32_t s = 0; s < res.n_slots; ++s)
        for (uint64_t i = 0; i < res.slots[s].n_values; ++i) sum += res.slots[s].values[i];
      printf("ok %llu signs digest %016llx\n", (unsigned long long)res.n_values_total, (unsigned long long)sum);
      fbxo_free(&res);
    } else {
      printf("status %d: %s\n", rc, err);
    }
  } else {
    uint8_t* out = NULL;
    uint64_t* out_off = NULL;
    uint64_t out_len = 0, kept = 0;
    rc = fbxo_clean((const char*)spec, spec_len, raw, raw_len, off, n, &out, &out_len, &out_off, &kept, err, sizeof err);
    if (rc == 0) {
      printf("ok %llu kept %llu bytes\n", (unsigned long long)kept, (unsigned long long)out_len);
      fbxo_clean_free(out, out_off);
    } else {
      printf("status %d: %s\n", rc, err);
    }
  }
  free(spec);
  free(raw);
  free(off_bytes);
  free(off);
  return 0;
}
