// Internal tables shared by the plan builder (host) and the HIP kernels.
#pragma once

#include <cstdint>
#include <vector>

#include "qv2.h"

namespace qv2 {

// Threads per workgroup of every tile kernel (8 wavefronts of 64).
#ifndef QV2_BLOCK
#define QV2_BLOCK 512
#endif
constexpr int kBlock = QV2_BLOCK;
// Largest row-group tile in elements: it is staged whole in LDS (32 KiB).
constexpr int kRowGroupCap = 8192;
// Most rows one row-group tile may hold.
constexpr int kRowGroupMaxRows = 1024;
// Default stream-tile length in elements (128 KiB of fp32).
constexpr int kDefaultTile = 32768;
// A segment (or pair tensor) with more partials than this is folded by a whole
// 1024-thread workgroup instead of one wavefront.
constexpr int kFoldWaveMax = 128;

struct TensorDesc {            // 48 B, device copy indexed by tensor
  const float* x;
  const float* qrun;
  int8_t* codes;
  int64_t numel;
  int32_t seg0;                // first segment of this tensor
  int32_t nseg;
  int32_t scheme;
  int32_t _pad;
};

// A tile is a contiguous element range of one tensor.
//  rows == 0 : stream tile, part of ONE segment (seg0); yields one partial (part0).
//  rows  > 0 : row-group tile, `rows` whole segments of `inner` elements each,
//              starting at segment seg0; yields `rows` partials from part0.
struct Tile {                  // 32 B
  int64_t off;                 // element offset inside the tensor
  int32_t len;                 // elements
  int32_t tensor;
  int32_t part0;
  int32_t rows;
  int32_t seg0;
  int32_t inner;
};

struct Segment {               // 24 B
  int64_t n;                   // elements in the segment
  int32_t part0;               // its partials, in element order
  int32_t nparts;
  int32_t scheme;
  int32_t _pad;
};

struct PairTensor {            // 16 B, one per tensor of the plan
  int64_t n;                   // 0 when the tensor has no qrun
  int32_t part0;
  int32_t nparts;
};

// Partial records the tile kernels leave in the workspace.
struct StatPartial { float mn, mx; double sx, sx2; };   // calibrate, 24 B
struct ErrPartial { double sx2, se2; };                 // fakequant and pair, 16 B
struct ErrPartial3 { double sx2, se2, sd2; };           // fused fakequant + pair, 24 B

}  // namespace qv2

struct qv2_plan {
  std::vector<qv2_tensor> tensors;
  std::vector<qv2::TensorDesc> descs;
  std::vector<qv2::Tile> tiles;          // stream tiles first, then row-group tiles
  std::vector<qv2::Segment> segments;
  std::vector<qv2::Tile> pair_tiles;     // stream tiles over tensors with qrun
  std::vector<qv2::PairTensor> pair_tensors;
  std::vector<int32_t> big_segments;      // segments with > kFoldWaveMax partials
  std::vector<int32_t> big_pair_tensors;  // pair tensors with > kFoldWaveMax partials
  // fused fake-quant + pair pass: a tensor's pair energy is folded from ALL its partial
  // slots of the main tile table (they are contiguous per tensor)
  std::vector<qv2::PairTensor> fused_pair_tensors;
  std::vector<int32_t> big_fused_pair_tensors;
  int64_t n_stream_tiles = 0;
  int64_t n_parts = 0;
  int32_t tile_elems = qv2::kDefaultTile;
  size_t workspace_bytes = 0;

  // device copy (made by the first device call, on the device current then)
  void* d_blob = nullptr;
  qv2::TensorDesc* d_descs = nullptr;
  qv2::Tile* d_tiles = nullptr;
  qv2::Segment* d_segments = nullptr;
  qv2::Tile* d_pair_tiles = nullptr;
  qv2::PairTensor* d_pair_tensors = nullptr;
  int32_t* d_big_segments = nullptr;
  int32_t* d_big_pair_tensors = nullptr;
  qv2::PairTensor* d_fused_pair_tensors = nullptr;
  int32_t* d_big_fused_pair_tensors = nullptr;

  // optional per-kernel timing (qv2_plan_set_timing): hipEvent_t handles
  bool timing = false;
  void* ev_start[QV2_K_COUNT] = {};
  void* ev_stop[QV2_K_COUNT] = {};
  bool ev_used[QV2_K_COUNT] = {};
};
