// Internal tables shared by the plan builder (host) and the HIP kernels.
#pragma once

#include <cstdint>
#include <vector>

#include "qv2.h"

// Compile-time tuning knobs (defaults are the measured best on MI355X).
#ifndef QV2_BLOCK_READ
#define QV2_BLOCK_READ 512     // threads of the read-only stream kernels (stats, pair)
#endif
#ifndef QV2_BLOCK_QUANT
#define QV2_BLOCK_QUANT 256    // threads of the quantize kernels (they also store codes)
#endif
#ifndef QV2_BLOCK_ROWS
#define QV2_BLOCK_ROWS 256     // threads of the row-group kernels (measured: 256 and 128 beat 512 by 10 %)
#endif
#ifndef QV2_VEC_QUANT
#define QV2_VEC_QUANT 2        // 16-byte loads per lane and stream in one batch of a quantize kernel
#endif

namespace qv2 {

constexpr int kBlockRead = QV2_BLOCK_READ;
constexpr int kBlockQuant = QV2_BLOCK_QUANT;
constexpr int kBlockRows = QV2_BLOCK_ROWS;
constexpr int kVecQuant = QV2_VEC_QUANT;

// Largest row-group tile in elements: it is staged whole in LDS (32 KiB).
constexpr int kRowGroupCap = 8192;
// Most rows one row-group tile may hold.
constexpr int kRowGroupMaxRows = 1024;
// ... and most rounds of the LDS-form row kernels one tile may take (a round = one row per lane
// group of every wavefront).  Short tiles keep the longest-running workgroup of the launch short:
// measured, a tile of 910 nine-element rows (29 rounds) alone made the MobileNetV2 launch twice as
// long as four-round tiles do, and one round is another 5-15 % better on all sets.
constexpr int kRowGroupRounds = 1;
// Register form of a row-group tile: a lane holds at most this many 16-byte vectors of its row
// and a row takes the smallest power-of-two number of lanes that can hold it (at least
// kRowRegMinLanes).  Measured on the VGG-16 and ResNet-50 weights: 16 vectors per lane (most
// rows then live in one wavefront, with 16 loads in flight per lane) beat 4, 8 and 32.
constexpr int kRowRegVecs = 16;
constexpr int kRowRegMinLanes = 16;
constexpr int kRowRegMinInner = 64;
static_assert(kBlockRows * 4 * kRowRegVecs >= kRowGroupCap, "a whole row must fit the registers of one workgroup");
// The register form also takes rows the LDS copy could not hold: up to kBlockRows * 64 elements
// with the row kernels' usual workgroup (one row per workgroup), and up to kRowRegCap with a
// workgroup of kBlockRowsWide threads.  A per-channel weight with rows that long (the first
// fully connected layer of VGG-16: 4096 rows of 25088) is then read from HBM once, too.
constexpr int kBlockRowsWide = 512;
// tiles per block of the XCD-aware tile order of the read-only sweeps (16 tiles of 32768 elements: 2 MB)
#ifndef QV2_XCD_BLOCK_READ
#define QV2_XCD_BLOCK_READ 16
#endif
constexpr int kXcdBlockRead = QV2_XCD_BLOCK_READ;
#ifndef QV2_XCD_BLOCK_QUANT
#define QV2_XCD_BLOCK_QUANT 256
#endif
constexpr int kXcdBlockQuant = QV2_XCD_BLOCK_QUANT;   // ... of the quantize sweeps (256 tiles of 2048 elements: 2 MB)
constexpr int kRowRegCap = kBlockRowsWide * 4 * kRowRegVecs;          // 32768 elements
// How a per-channel tensor's rows are handled.
enum RowForm { kRowStream = 0, kRowLds = 1, kRowReg = 2, kRowRegWide = 3 };
// Stream-tile length of the read-only passes (128 KiB of fp32): long tiles amortise the
// per-workgroup reduction.
constexpr int kDefaultReadTile = 32768;
// Stream-tile length of the quantize passes: exactly one batch per lane
// (block x kVecQuant x 4 elements).  A kernel that mixes code stores into the read stream
// runs fastest when all in-flight workgroups sweep a narrow address window.
constexpr int kDefaultQuantTile = kBlockQuant * kVecQuant * 4;
// Largest tensor a plan accepts: 2^36 elements (256 GiB of fp32, about all of the device memory); keeps
// the host tile tables of a nonsense length from being built at all.
constexpr int64_t kMaxNumel = int64_t{1} << 36;

// Histogram pass: a chunk is at least this long; the plan aims at about kHistChunks chunks.
constexpr int kHistMinChunk = 65536;
constexpr int kHistChunks = 4096;
constexpr int kHistMaxBins = 4096;
// A segment (or pair tensor) with more partials than this is folded by a whole
// 1024-thread workgroup instead of one wavefront.
constexpr int kFoldWaveMax = 128;

// Host code and kernels share the tile addressing below.
#if defined(__HIPCC__)
#define QV2_HD __host__ __device__
#else
#define QV2_HD
#endif

// A row-group tile (and a histogram chunk) is a contiguous element range of one tensor,
// addressed absolutely: a workgroup needs one 64-byte scalar load before it can issue its data loads.
//  rows  > 0 : row-group tile, `rows` whole segments of `inner` elements each,
//              starting at segment seg0; yields `rows` partials from part0.  Two forms: staged
//              in LDS (any alignment, any row length up to kRowGroupCap), or held in registers
//              (`lanes` > 0: rows of a multiple of 4 elements on 16-byte boundaries).
//  rows == 0 : a histogram chunk (part0 = chunk index), or a stream tile decoded from a Run.
struct Tile {                  // 64 B
  const float* x;              // first element of the tile
  const float* q;              // same position in the quantized-run tensor, or null
  int8_t* c;                   // same position in the code buffer, or null
  int32_t len;                 // elements
  int32_t part0;
  int32_t seg0;
  int32_t rows;
  int32_t inner;
  int32_t tensor;
  int32_t lanes;               // register-path row tiles: lanes that share one row (16 .. 512)
  int32_t _pad[3];
};
static_assert(sizeof(Tile) == 64, "Tile must stay one 64-byte record");

// Stream tiles (the sweeps over long segments) are not stored at all: a tensor's tiles form a
// Run, and workgroup k of a launch finds its tile by arithmetic.  A run's segments all have
// `inner` elements and are cut into `tiles_per_seg` tiles of `tile_len` elements (the last one of
// a segment shorter); tile j of the run belongs to segment seg0 + j / tiles_per_seg and owns
// partial slot part0 + j.  The tables a kernel touches before its data loads are therefore a few
// KB that stay in the scalar cache, instead of one 64-byte record per tile streamed from memory
// (85 MB for the 1.3 M quantize tiles of the ResNet-50 batch-256 activations).
struct Run {                   // 64 B, one per tensor of a stream-tile table
  const float* x;              // first element of the tensor
  const float* q;              // ... of its quantized-run partner, or null
  int8_t* c;                   // ... of its code buffer, or null
  int64_t inner;               // elements per segment
  int32_t tile0;               // index of the run's first tile in the launch
  int32_t tiles_per_seg;
  int32_t seg0;                // first segment of the tensor
  int32_t part0;               // partial slot of the run's first tile
  int32_t tile_len;
  int32_t tensor;
  int32_t tile_end;            // tile0 + number of tiles: a record says by itself whether it holds tile k
  int32_t _pad;
};
static_assert(sizeof(Run) == 64, "Run must stay one 64-byte record");

// What a kernel is handed: the runs in launch order, and for every block of 2^shift consecutive
// tile indices the run that holds the block's first tile (so the search is one lookup and, where
// a block spans several small tensors, a short walk).
struct StreamView {
  const Run* runs;
  const int32_t* coarse;
  int32_t n_runs;
  int32_t shift;
};

struct TileRef {               // one decoded stream tile
  const float* x;
  const float* q;
  int8_t* c;
  int32_t len, part0, seg0, tensor;
};

// Workgroups go to the 8 XCDs of the chip in turn (workgroup k runs on XCD k mod 8).  With
// tiles handed out in table order every XCD touches every eighth tile; this mapping instead lets
// each XCD work through blocks of `block` neighbouring tiles, the 8 XCDs on 8 neighbouring blocks,
// so the tiles in flight on the whole chip still form one window.  A permutation of 0 .. n-1: the
// tiles past the last whole group of 8 blocks keep their places.  Measured on the calibration
// sweep with blocks of 2 MB of x: -2 % on the ResNet-50 batch-256 set, no change on the smallest set.
QV2_HD inline int xcd_blocked(int k, int n, int block) {
  const int group = k / (8 * block);
  if ((group + 1) * 8 * block > n) return k;
  const int in = k - group * 8 * block;          // XCD = in & 7, place in its block = in >> 3
  return group * 8 * block + (in & 7) * block + (in >> 3);
}

// A workgroup sits idle until this has run, so its chain of dependent scalar loads and its
// arithmetic are part of every tile's time.  Two forms, same result.  The default one walks whole
// records (table entry, then record: two dependent loads in the usual case) and skips the
// division for a run that is one segment (every per-tensor scheme): 5-7 % on the quantize sweeps
// that also sum x^2 or compare with qrun.  PLAIN is the earlier form - the walk looks at the next
// record's first tile, the division always runs -, which the quantize sweep of the single call (error
// energy only) prefers by 1.7 %, measured both ways on the ResNet-50 batch-256 set.
template <bool PLAIN = false>
QV2_HD inline TileRef decode_tile(const StreamView& v, int32_t k) {
  int32_t r = v.coarse[k >> v.shift];
  Run rn;
  if (PLAIN) {
    while (r + 1 < v.n_runs && v.runs[r + 1].tile0 <= k) ++r;
    rn = v.runs[r];
  } else {
    rn = v.runs[r];
    while (k >= rn.tile_end && r + 1 < v.n_runs) rn = v.runs[++r];
  }
  const int32_t j = k - rn.tile0;
  const int32_t s = (PLAIN || j >= rn.tiles_per_seg) ? j / rn.tiles_per_seg : 0, i = j - s * rn.tiles_per_seg;
  const int64_t in_seg = static_cast<int64_t>(i) * rn.tile_len;
  const int64_t off = static_cast<int64_t>(s) * rn.inner + in_seg;
  const int64_t left = rn.inner - in_seg;
  TileRef t;
  t.x = rn.x + off;
  t.q = rn.q ? rn.q + off : nullptr;
  t.c = rn.c ? rn.c + off : nullptr;
  t.len = static_cast<int32_t>(left < rn.tile_len ? left : rn.tile_len);
  t.part0 = rn.part0 + j;
  t.seg0 = rn.seg0 + s;
  t.tensor = rn.tensor;
  return t;
}

// Host side of a stream-tile table.
struct StreamTable {
  std::vector<Run> runs;
  std::vector<int32_t> coarse;
  int32_t shift = 0;
  int64_t n_tiles = 0;
  StreamView view() const {
    return StreamView{runs.data(), coarse.data(), static_cast<int32_t>(runs.size()), shift};
  }
  // all tiles, decoded the way the kernels decode them (tests, diagnostics)
  std::vector<Tile> expand() const {
    std::vector<Tile> out;
    out.reserve(static_cast<size_t>(n_tiles));
    const StreamView v = view();
    for (int64_t k = 0; k < n_tiles; ++k) {
      const TileRef r = decode_tile(v, static_cast<int32_t>(k));
      const TileRef r2 = decode_tile<true>(v, static_cast<int32_t>(k));       // the other form: same tile
      if (r.x != r2.x || r.q != r2.q || r.c != r2.c || r.len != r2.len || r.part0 != r2.part0 ||
          r.seg0 != r2.seg0 || r.tensor != r2.tensor) return std::vector<Tile>();
      Tile t{};
      t.x = r.x; t.q = r.q; t.c = r.c; t.len = r.len; t.part0 = r.part0; t.seg0 = r.seg0; t.tensor = r.tensor;
      out.push_back(t);
    }
    return out;
  }
};
// Most entries a coarse table may have (it is sized to the launch: 2^shift tiles per entry).
constexpr int64_t kCoarseMax = 2048;

// Partial slots come in two numberings: `sp` for the calibration pass (read tiles) and
// `ep` for the quantize passes (quantize tiles).  Row-group partials have the same index
// in both (they come first); stream partials follow.
struct Segment {               // 32 B
  int64_t n;                   // elements in the segment
  int32_t sp0, snp;            // calibration partials, in element order
  int32_t ep0, enp;            // quantize partials, in element order
  int32_t scheme;
  int32_t tensor;              // the tensor the segment belongs to
};

struct PairTensor {            // 16 B, one per tensor of the plan
  int64_t n;                   // 0 when the tensor has no qrun
  int32_t part0;
  int32_t nparts;
};

struct HistTensor {            // 16 B, one per tensor: its chunks of the histogram pass
  int32_t chunk0, nchunks;
  int32_t seg0, nseg;
};

struct TensorInfo {            // host only
  int64_t numel;
  int32_t seg0, nseg;
  int32_t kind, layer;         // as given in the layer table (route results to per-layer series)
  bool has_pair;
};

// Partial records the tile kernels leave in the workspace.
struct StatPartial { float mn, mx; double sx, sx2; };   // calibrate, 24 B
struct StatPairPartial { float mn, mx; double sx, sx2, sd2; };  // calibrate + pair comparison, 32 B
struct StatPairCosPartial { float mn, mx; double sx, sx2, sd2, sxq; };  // ... + cosine cross term, 40 B
struct ErrPartial { double sx2, se2; };                 // pair pass, 16 B
struct ErrPartial1 { double se2; };                     // quantize sweep of a whole pass (the other energies
                                                        // were taken by its first sweep), 8 B
struct ErrPartial3 { double sx2, se2, sd2; };           // quantize passes, 24 B
struct ErrPartial5 { double sx2, se2, sd2, sxh, sxq; }; // quantize pass with cosine cross terms, 40 B

}  // namespace qv2

struct qv2_plan {
  std::vector<qv2::TensorInfo> info;
  qv2::StreamTable read_tiles;           // calibration: stream tiles (read size)
  qv2::StreamTable quant_tiles;          // quantize passes: stream tiles (quantize size)
  qv2::StreamTable quant_ro_tiles;       // ... of tensors without a code buffer: the sweep only reads
                                         // them, so they are cut like the read-only passes' tiles
  std::vector<qv2::Tile> row_tiles;      // row-group tiles staged in LDS, used by both
  std::vector<qv2::Tile> reg_tiles;      // row-group tiles held in registers, used by both
  std::vector<qv2::Tile> wide_tiles;     // ... one long row each, held by a workgroup of kBlockRowsWide threads
  int64_t n_single_read = 0;             // elements of the tensors made of row-group tiles
  qv2::StreamTable pair_tiles;           // pair pass: stream tiles over tensors with qrun
  std::vector<qv2::Tile> hist_tiles;     // histogram pass: long chunks (part0 = chunk index)
  std::vector<qv2::HistTensor> hist_tensors;
  std::vector<qv2::Segment> segments;
  std::vector<qv2::PairTensor> pair_tensors;        // partial ranges of the pair pass
  std::vector<qv2::PairTensor> fused_pair_tensors;  // ranges in the quantize numbering
  std::vector<qv2::PairTensor> stat_pair_tensors;   // ranges in the calibration numbering; only
                                                    // tensors made of stream tiles (n = 0 otherwise)
  std::vector<int32_t> big_stat_segments;   // segments with > kFoldWaveMax calibration partials
  std::vector<int32_t> big_err_segments;    // ... quantize partials
  std::vector<int32_t> big_pair_tensors;
  std::vector<int32_t> big_fused_pair_tensors;
  std::vector<int32_t> big_stat_pair_tensors;
  // per-tensor records made inside the last fold of a pass instead of by a launch of their own:
  std::vector<int32_t> row_tensors;         // tensors made of row-group tiles (their segment records are
                                            // final when that fold starts): one workgroup each
  std::vector<int32_t> late_tensors;        // tensors of several stream segments, whose records that same
                                            // fold launch only just writes: a small launch after it
  int32_t read_tile = qv2::kDefaultReadTile;
  int32_t quant_tile = qv2::kDefaultQuantTile;
  bool rows_have_pair = false;           // some row-group tensor has a quantized-run partner
  int32_t n_row_parts = 0;               // partial slots 0 .. n_row_parts-1 belong to row-group segments
  size_t workspace_bytes = 0;

  // device copy (made by the first device call, on the device current then)
  void* d_blob = nullptr;
  int device = -1;               // the device that holds d_blob (current at the first device call)
  qv2::StreamView d_read_tiles = {};     // device views of the four stream-tile tables
  qv2::StreamView d_quant_tiles = {};
  qv2::StreamView d_quant_ro_tiles = {};
  qv2::StreamView d_pair_tiles = {};
  qv2::Tile* d_row_tiles = nullptr;
  qv2::Tile* d_reg_tiles = nullptr;
  qv2::Tile* d_wide_tiles = nullptr;
  qv2::Tile* d_hist_tiles = nullptr;
  qv2::HistTensor* d_hist_tensors = nullptr;
  qv2::Segment* d_segments = nullptr;
  qv2::PairTensor* d_pair_tensors = nullptr;
  qv2::PairTensor* d_fused_pair_tensors = nullptr;
  qv2::PairTensor* d_stat_pair_tensors = nullptr;
  int32_t* d_big_stat_segments = nullptr;
  int32_t* d_big_err_segments = nullptr;
  int32_t* d_big_pair_tensors = nullptr;
  int32_t* d_big_fused_pair_tensors = nullptr;
  int32_t* d_big_stat_pair_tensors = nullptr;
  int32_t* d_row_tensors = nullptr;
  int32_t* d_late_tensors = nullptr;

  // optional per-kernel timing (qv2_plan_set_timing): hipEvent_t handles
  bool timing = false;
  void* ev_start[QV2_K_COUNT] = {};
  void* ev_stop[QV2_K_COUNT] = {};
  bool ev_used[QV2_K_COUNT] = {};
  int time_only = -1;            // >= 0: only this kernel's launches are bracketed
  // completion marks of the two passes qv2_sensitivity_pass_begin may have in flight
  void* ev_done[2] = {};
};
