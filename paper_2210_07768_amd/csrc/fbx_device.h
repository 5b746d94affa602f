// Kernel parameter block and launch wrappers shared by the kernels and the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include "fbx_internal.h"

namespace fbx {

constexpr int kBlock = 256;  // threads per workgroup of the tile, scan and allocation kernels

struct TileParams {
  const uint8_t* raw;
  uint64_t raw_len;
  const uint64_t* rec_off;
  uint64_t n_records;
  uint8_t* ws;  // workspace base
  const OpDesc* ops;
  const uint32_t* layer_ops;
  const uint32_t* layer_begin;
  const uint32_t* nonroot;
  const uint8_t* aux;
  OpDyn* dyn;
  Ctrl* ctrl;
  uint32_t* tile_cnt;   // [n_ragged][n_tiles]
  uint64_t* tile_base;  // [n_ragged][n_tiles]
  uint32_t n_ops, n_layers, n_ragged, n_nonroot;
  uint32_t n_tiles, log2T, n_fields;
  uint32_t layer_lo, layer_hi;  // 1-based, inclusive
  uint32_t cap_bytes, cap_tabs;
  uint32_t lds_cnt, lds_tab, lds_mask, lds_bytes;  // byte offsets into dynamic LDS
};

hipError_t launch_reset(Ctrl* ctrl, uint64_t arena_base, hipStream_t st);
hipError_t launch_validate(const uint64_t* rec_off, uint64_t n_records, uint64_t raw_len, uint32_t log2T, Ctrl* ctrl,
                           hipStream_t st);
hipError_t launch_tile(const TileParams& P, bool count, uint32_t lds_bytes, hipStream_t st);
hipError_t launch_scan(const uint32_t* tile_cnt, uint64_t* tile_base, uint64_t* row_total, uint32_t n_ragged,
                       uint32_t n_tiles, const Ctrl* ctrl, hipStream_t st);
hipError_t launch_alloc(const OpDesc* ops, OpDyn* dyn, uint32_t n_ops, uint32_t n_layers, const uint64_t* row_total,
                        uint64_t n_records, uint64_t ws_bytes, uint8_t* ws, int reuse, Ctrl* ctrl, hipStream_t st);
hipError_t launch_arena_alloc(uint64_t* head, const uint64_t* sizes, uint64_t n, uint64_t* offsets, uint32_t threads,
                              hipStream_t st);
hipError_t launch_arena_reset(uint64_t* head, uint64_t value, hipStream_t st);

}  // namespace fbx
