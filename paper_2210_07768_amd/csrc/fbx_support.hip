// Support kernels of libfbx: per-call reset and input validation, the scan that
// turns per-tile counts into per-tile bases, and the arena (Algorithm 1 of the
// paper and the per-call carving of operator arrays).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "fbx_arena.h"
#include "fbx_device.h"

namespace fbx {

// --------------------------------------------------------------- validation
__global__ void k_reset(Ctrl* ctrl, uint64_t arena_base) {
  if (threadIdx.x == 0) {
    ctrl->err = 0; ctrl->pad0 = 0; ctrl->required = 0; ctrl->head = arena_base; ctrl->high_water = arena_base;
    ctrl->n_malformed = 0; ctrl->max_tile_bytes = 0; ctrl->slow_tiles = 0; ctrl->ticket[0] = 0; ctrl->ticket[1] = 0;
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
      // the maximum only ever grows: skip the atomic unless this tile can raise it
      if (hi - a > *reinterpret_cast<volatile uint64_t*>(&ctrl->max_tile_bytes))
        atomicMax(reinterpret_cast<unsigned long long*>(&ctrl->max_tile_bytes), (unsigned long long)(hi - a));
    }
  }
  if (err) atomicOr(&ctrl->err, err);
}

// --------------------------------------------------------------------- scan
// Exclusive scan over tiles of every ragged operator's per-tile counts, in two launches.  A row
// (one operator) is cut into segments of kScanSeg tiles; a workgroup takes one segment of one
// row.  k_scan_sums adds its segment up; k_scan adds the sums of the segments before its own
// (its carry), then scans its segment 256 tiles at a time.  Neighbouring lanes read and write
// neighbouring entries throughout.
__device__ __forceinline__ uint64_t block_sum(uint64_t v, uint64_t* s) {  // s: kBlock / 64 entries; every lane gets the sum
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  const uint32_t w = threadIdx.x >> 6;
  __syncthreads();  // (s may still be read from an earlier call)
  if ((threadIdx.x & 63u) == 0) s[w] = v;
  __syncthreads();
  uint64_t t = 0;
  for (uint32_t i = 0; i < kBlock / 64; ++i) t += s[i];
  return t;
}

__global__ __launch_bounds__(kBlock) void k_scan_sums(const uint32_t* tile_cnt, uint64_t* part, uint32_t n_tiles,
                                                      uint32_t n_seg, const Ctrl* ctrl) {
  __shared__ uint64_t s[kBlock / 64];
  if (ctrl->err) return;
  const uint32_t row = blockIdx.x / n_seg, seg = blockIdx.x % n_seg, tid = threadIdx.x;
  const uint32_t* src = tile_cnt + (uint64_t)row * n_tiles;
  const uint32_t lo = seg * kScanSeg, hi = min(lo + kScanSeg, n_tiles);
  uint64_t sum = 0;
  for (uint32_t i = lo + tid; i < hi; i += kBlock) sum += src[i];
  sum = block_sum(sum, s);
  if (tid == 0) part[(uint64_t)row * n_seg + seg] = sum;
}

__global__ __launch_bounds__(kBlock) void k_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total,
                                                 const uint64_t* part, uint32_t n_tiles, uint32_t n_seg, const Ctrl* ctrl) {
  __shared__ uint64_t s[kBlock / 64];
  __shared__ uint64_t s_wave[kBlock / 64];
  if (ctrl->err) return;
  const uint32_t row = blockIdx.x / n_seg, seg = blockIdx.x % n_seg, tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t* src = tile_cnt + (uint64_t)row * n_tiles;
  uint64_t* dst = tile_base + (uint64_t)row * n_tiles;
  uint64_t before = 0;
  for (uint32_t i = tid; i < seg; i += kBlock) before += part[(uint64_t)row * n_seg + i];
  uint64_t carry = block_sum(before, s);
  const uint32_t lo = seg * kScanSeg, hi = min(lo + kScanSeg, n_tiles);
  for (uint32_t i0 = lo; i0 < hi; i0 += kBlock) {
    const uint32_t i = i0 + tid;
    const uint64_t v = i < hi ? src[i] : 0u;
    uint64_t incl = v;
    for (int d = 1; d < 64; d <<= 1) {
      const uint64_t t = __shfl_up(incl, d, 64);
      if (lane >= (uint32_t)d) incl += t;
    }
    __syncthreads();  // (s_wave of the step before has been read)
    if (lane == 63u) s_wave[wave] = incl;
    __syncthreads();
    uint64_t below = 0, all = 0;
    for (uint32_t w = 0; w < kBlock / 64; ++w) {
      const uint64_t t = s_wave[w];
      if (w < wave) below += t;
      all += t;
    }
    if (i < hi) dst[i] = carry + below + incl - v;
    carry += all;
  }
  if (seg + 1u == n_seg && tid == 0) row_total[row] = carry;
}

// ------------------------------------------------------------------- arena
// (Algorithm 1 itself, arena_alloc_wg, lives in fbx_arena.h: any kernel can call it)
__device__ __forceinline__ uint64_t round128(uint64_t x) { return arena_round128(x); }

__global__ void k_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets) {
  __shared__ uint64_t s_part[1024 / 64 + 2];
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t size = i < n ? sizes[i] : 0;
  const uint64_t off = arena_alloc_wg(head, size, s_part);
  if (i < n) offsets[i] = off;
}

__global__ void k_arena_reset(uint64_t* head, uint64_t value) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *head = value;
}

// Flattened per-call programs: everything a kernel needs about an operator (or
// about a single-valued hash field) in one aligned record.  One block of kBlock threads.
__device__ void write_programs(const WalkParams& P, bool placed) {
  const OpDesc* ops = P.ops;
  const OpDyn* dyn = P.dyn;
  const uint64_t origin = P.origin;
  const uint32_t tid = threadIdx.x;
  __syncthreads();
  for (uint32_t i = tid; i < P.n_ops; i += kBlock) {
    const OpDesc& d = ops[i];
    OpProg g;
    g.kind = d.kind; g.flags = d.flags; g.arity = d.arity; g.rag_row = d.rag_row;
    g.aux_off = d.aux_off; g.aux_len = d.aux_len; g.a = d.a; g.b = d.b;
    g.key = d.key;
    g.values = placed ? origin + dyn[i].values_off : 0;
    g.offsets = (placed && !d.arity) ? origin + dyn[i].offsets_off : 0;
    g.field = d.field;
    g.stage = d.stage;
    if (d.kind == OP_CROSS && ops[d.a].arity == 1 && ops[d.b].arity == 1) {
      // a cross of two single signs finds both in the on-chip table: rows instead of aux data
      g.aux_off = ops[d.a].stage;
      g.aux_len = ops[d.b].stage;
    }
    if (d.kind == OP_CROSS && d.fuse) {
      // a cross computed along with its multi-valued hash: the other input's row, and which side the hash is on
      g.aux_off = ops[d.fuse == 1 ? d.b : d.a].stage;
      g.aux_len = d.fuse == 1 ? 1u : 0u;
    }
    if (d.kind == OP_HASH && !d.arity) {  // a multi-valued hash: its crosses of that kind (first, number)
      g.a = d.fuse & 0xffffu;
      g.b = d.fuse >> 16;
    }
    P.prog_ops[i] = g;
  }
  for (uint32_t k = tid; k < P.n_fields; k += kBlock) {
    const FieldDesc& f = P.fields[k];
    FieldProg g;
    g.cls = f.cls; g.need = f.need; g.op_begin = f.op_begin; g.op_count = f.op_count;
    g.key = 0; g.dst = 0;
    if (f.cls == FC_HASH1) {
      const uint32_t op = P.field_ops[f.op_begin];
      g.key = ops[op].key;
      g.dst = placed ? origin + dyn[op].values_off : 0;
    }
    P.prog_fields[k] = g;
  }
}

// Carve the operators' value / offset arrays out of the pool, once sizes are
// known.  Emitted operators first (they live until the next call); then layer
// by layer the intermediates born in that layer, and after each layer the head
// drops back as far as still-live intermediates allow: the constant-time reset
// of Section 5 ("Reset GPU memory pool"), generalised to outputs that a later
// layer still reads.  With reuse off (all layers in one launch) nothing is
// released.  One block of kBlock threads.
__global__ __launch_bounds__(kBlock) void k_alloc(WalkParams P, const uint64_t* row_total, uint64_t ws_bytes, int reuse) {
  const OpDesc* ops = P.ops;
  OpDyn* dyn = P.dyn;
  Ctrl* ctrl = P.ctrl;
  const uint32_t n_ops = P.n_ops, n_layers = P.n_layers;
  const uint64_t n_records = P.n_records;
  __shared__ uint64_t s_part[kBlock / 64 + 2];
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
      const uint64_t off = arena_alloc_wg(&ctrl->head, sv + so, s_part);
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
      if (!ops[i].arity) *reinterpret_cast<uint64_t*>(P.origin + dyn[i].offsets_off) = 0;
  }
  write_programs(P, true);
}

// The per-call programs alone, without placement (array addresses are left zero):
// all the counting launch of the tile kernel needs.
__global__ __launch_bounds__(kBlock) void k_programs(WalkParams P) { write_programs(P, false); }

__global__ void k_fill64(uint64_t* p, uint64_t n, uint64_t value) {
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) p[i] = value;
}

// An empty kernel with five pointer arguments: what Table 1 of the paper launches to measure the
// launch overhead that motivates one meta-kernel per layer (Section 4).
__global__ void k_empty(const void*, const void*, const void*, const void*, void*) {}

hipError_t launch_empty(uint32_t n, hipStream_t st) {
  for (uint32_t i = 0; i < n; ++i) {
    hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, st, (const void*)nullptr, (const void*)nullptr, (const void*)nullptr,
                       (const void*)nullptr, (void*)nullptr);
  }
  return hipGetLastError();
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

uint32_t scan_segments(uint32_t n_tiles) { return n_tiles ? (n_tiles + kScanSeg - 1u) / kScanSeg : 1u; }

hipError_t launch_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total, uint64_t* part, uint32_t n_ragged,
                       uint32_t n_tiles, const Ctrl* ctrl, hipStream_t st) {
  if (n_ragged == 0) return hipSuccess;
  const uint32_t n_seg = scan_segments(n_tiles);
  if (n_seg > 1u) {  // (one segment a row: nothing lies before it)
    hipLaunchKernelGGL(k_scan_sums, dim3(n_ragged * n_seg), dim3(kBlock), 0, st, tile_cnt, part, n_tiles, n_seg, ctrl);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_scan, dim3(n_ragged * n_seg), dim3(kBlock), 0, st, tile_cnt, tile_base, row_total, part, n_tiles, n_seg,
                     ctrl);
  return hipGetLastError();
}

hipError_t launch_alloc(const WalkParams& P, const uint64_t* row_total, uint64_t ws_bytes, int reuse, hipStream_t st) {
  hipLaunchKernelGGL(k_alloc, dim3(1), dim3(kBlock), 0, st, P, row_total, ws_bytes, reuse);
  return hipGetLastError();
}

hipError_t launch_fill64(uint64_t* p, uint64_t n, uint64_t value, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const uint32_t blocks = (uint32_t)std::min<uint64_t>((n + 255) / 256, 8192);
  hipLaunchKernelGGL(k_fill64, dim3(blocks), dim3(256), 0, st, p, n, value);
  return hipGetLastError();
}

hipError_t launch_programs(const WalkParams& P, hipStream_t st) {
  hipLaunchKernelGGL(k_programs, dim3(1), dim3(kBlock), 0, st, P);
  return hipGetLastError();
}

hipError_t launch_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets, uint32_t threads,
                              hipStream_t st) {
  if (n == 0) return hipSuccess;
  const uint64_t blocks = (n + threads - 1) / threads;
  hipLaunchKernelGGL(k_arena_alloc, dim3((uint32_t)blocks), dim3(threads), 0, st, head, sizes, n, offsets);
  return hipGetLastError();
}

hipError_t launch_arena_reset(uint64_t* head, uint64_t value, hipStream_t st) {
  hipLaunchKernelGGL(k_arena_reset, dim3(1), dim3(64), 0, st, head, value);
  return hipGetLastError();
}

}  // namespace fbx
