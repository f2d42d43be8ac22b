// Host-only checks of the plan builder and the host functions of the qv2 C ABI, meant to be
// built with -fsanitize=address,undefined (tests/test_host_sanitize.py does that) and linked
// with csrc/qv2_host.cpp alone: no GPU, no HIP.  It builds many layer tables and verifies the
// invariants the kernels rely on (every element covered exactly once by every tile table - the
// stream tiles decoded from their runs by the very function the kernels use -, partial slots
// unique and inside the workspace, fold lists complete), then drives finalize, rank, BOPs,
// KL and regrouping over random and hostile inputs.  Prints "host checks ok" and exits 0.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <map>
#include <random>
#include <string>
#include <vector>

#include "qv2_internal.h"

#define CHECK(c)                                                              \
  do {                                                                        \
    if (!(c)) {                                                               \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
      std::exit(1);                                                           \
    }                                                                         \
  } while (0)

namespace {

using qv2::Segment;
using qv2::Tile;

// fake device addresses: never dereferenced by host code
float* fake_f32(uint64_t k) { return reinterpret_cast<float*>(0x100000000ull + k * 4); }
int8_t* fake_i8(uint64_t k) { return reinterpret_cast<int8_t*>(0x9000000000ull + k); }

struct Span { const float* x; int64_t len; };

// The tiles of one table that belong to tensor t must cover [x, x + numel) exactly once.
void check_cover(const std::vector<const std::vector<Tile>*>& tables, const qv2_tensor& in, int32_t t,
                 bool must_exist) {
  std::vector<Span> spans;
  for (const auto* tab : tables)
    for (const Tile& tl : *tab)
      if (tl.tensor == t) {
        CHECK(tl.len > 0);
        CHECK((tl.q == nullptr) == (in.qrun == nullptr));
        CHECK((tl.c == nullptr) == (in.codes == nullptr));
        const int64_t off = tl.x - in.x;
        if (in.qrun) CHECK(tl.q == in.qrun + off);
        if (in.codes) CHECK(tl.c == in.codes + off);
        spans.push_back({tl.x, tl.len});
      }
  if (!must_exist && spans.empty()) return;
  std::sort(spans.begin(), spans.end(), [](const Span& a, const Span& b) { return a.x < b.x; });
  const float* at = in.x;
  for (const Span& s : spans) {
    CHECK(s.x == at);
    at += s.len;
  }
  CHECK(at == in.x + in.numel);
}

// A stream-tile table as the kernels see it: workgroup k decodes tile k from the runs.
std::vector<Tile> decoded(const qv2::StreamTable& tab, int64_t block) {
  CHECK(tab.n_tiles >= 0 && tab.n_tiles * block <= int64_t{0xFFFFFFFF});        // one launch
  CHECK(tab.shift >= 0 && static_cast<int64_t>(tab.coarse.size()) == (tab.n_tiles >> tab.shift) + 1);
  CHECK(static_cast<int64_t>(tab.coarse.size()) <= qv2::kCoarseMax);
  int64_t at = 0;
  for (size_t r = 0; r < tab.runs.size(); ++r) {
    const qv2::Run& rn = tab.runs[r];
    CHECK(rn.tile0 == at && rn.tiles_per_seg > 0 && rn.tile_len > 0 && rn.inner > 0);
    CHECK(rn.tiles_per_seg == (rn.inner + rn.tile_len - 1) / rn.tile_len);
    at += r + 1 < tab.runs.size() ? tab.runs[r + 1].tile0 - rn.tile0 : tab.n_tiles - rn.tile0;
    CHECK((at - rn.tile0) % rn.tiles_per_seg == 0 && at > rn.tile0 && rn.tile_end == at);
  }
  CHECK(at == tab.n_tiles);
  for (size_t b = 0; b < tab.coarse.size() && !tab.runs.empty(); ++b) {
    // the walk from the coarse entry must start at or before the right run
    const int32_t r = tab.coarse[b];
    CHECK(r >= 0 && r < static_cast<int32_t>(tab.runs.size()));
    CHECK(tab.runs[r].tile0 <= static_cast<int64_t>(b) << tab.shift || r == 0);
  }
  std::vector<Tile> out = tab.expand();              // decodes every tile both ways; empty if they differ
  CHECK(static_cast<int64_t>(out.size()) == tab.n_tiles);
  return out;
}

void check_plan(const std::vector<qv2_tensor>& rows) {
  qv2_plan* p = nullptr;
  CHECK(qv2_plan_create(rows.data(), static_cast<int32_t>(rows.size()), &p) == QV2_OK);
  CHECK(p != nullptr);
  const std::vector<Tile> read_tiles = decoded(p->read_tiles, qv2::kBlockRead);
  const std::vector<Tile> quant_tiles = decoded(p->quant_tiles, qv2::kBlockQuant);
  const std::vector<Tile> quant_ro_tiles = decoded(p->quant_ro_tiles, qv2::kBlockRead);
  const std::vector<Tile> pair_tiles = decoded(p->pair_tiles, qv2::kBlockRead);
  const int32_t nt = static_cast<int32_t>(rows.size());
  CHECK(qv2_plan_num_tensors(p) == nt);
  CHECK(static_cast<int32_t>(p->info.size()) == nt);
  CHECK(static_cast<int32_t>(p->pair_tensors.size()) == nt);
  CHECK(static_cast<int32_t>(p->fused_pair_tensors.size()) == nt);
  CHECK(static_cast<int32_t>(p->hist_tensors.size()) == nt);

  int64_t nseg = 0;
  for (int32_t t = 0; t < nt; ++t) {
    const qv2_tensor& in = rows[t];
    CHECK(qv2_plan_segment_begin(p, t) == nseg);
    CHECK(p->info[t].seg0 == nseg);
    const int64_t s = in.scheme == QV2_SYM_CHANNEL ? in.channels : 1;
    CHECK(p->info[t].nseg == s && p->info[t].numel == in.numel);
    for (int64_t k = 0; k < s; ++k) {
      CHECK(p->segments[nseg + k].n == in.numel / s);
      CHECK(p->segments[nseg + k].scheme == in.scheme);
    }
    nseg += s;
    check_cover({&read_tiles, &p->row_tiles, &p->reg_tiles, &p->wide_tiles}, in, t, true);
    check_cover({&quant_tiles, &quant_ro_tiles, &p->row_tiles, &p->reg_tiles, &p->wide_tiles}, in, t, true);
    check_cover({&p->hist_tiles}, in, t, true);
    check_cover({&pair_tiles}, in, t, in.qrun != nullptr);
    if (!in.qrun) {
      for (const Tile& tl : pair_tiles) CHECK(tl.tensor != t);
      CHECK(p->pair_tensors[t].n == 0 && p->fused_pair_tensors[t].n == 0);
    } else {
      CHECK(p->pair_tensors[t].n == in.numel && p->fused_pair_tensors[t].n == in.numel);
    }
  }
  CHECK(qv2_plan_num_segments(p) == nseg);
  CHECK(static_cast<int64_t>(p->segments.size()) == nseg);
  CHECK(qv2_plan_num_tiles(p) ==
        static_cast<int64_t>(read_tiles.size() + p->row_tiles.size() + p->reg_tiles.size() + p->wide_tiles.size()));
  CHECK(qv2_plan_num_quant_tiles(p) ==
        static_cast<int64_t>(quant_tiles.size() + quant_ro_tiles.size() + p->row_tiles.size() + p->reg_tiles.size() +
                             p->wide_tiles.size()));
  CHECK(qv2_plan_num_pair_tiles(p) == static_cast<int64_t>(pair_tiles.size()));

  // partial slots: every slot of a numbering is written by exactly one (tile, row), lies in
  // its segment's range and inside the workspace
  const size_t ws = qv2_workspace_bytes(p);
  CHECK(ws % 256 == 0 && ws >= 256);
  std::vector<int> hits_s(ws / sizeof(qv2::StatPartial) + 1, 0), hits_e(ws / sizeof(qv2::ErrPartial5) + 1, 0);
  auto mark = [&](const Tile& tl, bool stats, bool quant) {
    CHECK(tl.seg0 >= 0 && tl.seg0 < nseg);
    if (tl.rows > 0) {
      CHECK(static_cast<int64_t>(tl.rows) * tl.inner == tl.len);
      if (tl.lanes == 0) CHECK(tl.len <= qv2::kRowGroupCap && tl.rows <= qv2::kRowGroupMaxRows);   // LDS copy
      else CHECK(tl.len <= qv2::kRowRegCap && tl.inner <= qv2::kRowRegCap);
      CHECK(tl.seg0 + tl.rows <= nseg);
      CHECK(tl.part0 + tl.rows <= p->n_row_parts);
      for (int r = 0; r < tl.rows; ++r) {
        const Segment& sg = p->segments[tl.seg0 + r];
        CHECK(sg.sp0 == tl.part0 + r && sg.snp == 1 && sg.ep0 == tl.part0 + r && sg.enp == 1);
        if (stats) { CHECK(static_cast<size_t>(tl.part0 + r) < hits_s.size() - 1); ++hits_s[tl.part0 + r]; }
        if (quant) { CHECK(static_cast<size_t>(tl.part0 + r) < hits_e.size() - 1); ++hits_e[tl.part0 + r]; }
      }
    } else {
      const Segment& sg = p->segments[tl.seg0];
      if (stats) {
        CHECK(tl.part0 >= sg.sp0 && tl.part0 < sg.sp0 + sg.snp && tl.part0 >= p->n_row_parts);
        CHECK(static_cast<size_t>(tl.part0) < hits_s.size() - 1);
        ++hits_s[tl.part0];
      }
      if (quant) {
        CHECK(tl.part0 >= sg.ep0 && tl.part0 < sg.ep0 + sg.enp && tl.part0 >= p->n_row_parts);
        CHECK(static_cast<size_t>(tl.part0) < hits_e.size() - 1);
        ++hits_e[tl.part0];
      }
    }
  };
  for (const Tile& tl : read_tiles) { CHECK(tl.rows == 0 && tl.len <= p->read_tile); mark(tl, true, false); }
  for (const Tile& tl : quant_tiles) { CHECK(tl.rows == 0 && tl.len <= p->quant_tile && tl.c); mark(tl, false, true); }
  for (const Tile& tl : quant_ro_tiles) { CHECK(tl.rows == 0 && tl.len <= p->read_tile && !tl.c); mark(tl, false, true); }
  for (const Tile& tl : p->row_tiles) { CHECK(tl.rows > 0 && tl.lanes == 0); mark(tl, true, true); }
  for (int wide = 0; wide < 2; ++wide)
  for (const Tile& tl : wide ? p->wide_tiles : p->reg_tiles) {
    // register form: whole vectors on 16-byte boundaries, a row fits its lanes, the rows fit the workgroup
    const int block = wide ? qv2::kBlockRowsWide : qv2::kBlockRows;
    CHECK(tl.rows > 0 && tl.inner % 4 == 0 && tl.inner >= qv2::kRowRegMinInner);
    CHECK(tl.lanes >= qv2::kRowRegMinLanes && tl.lanes <= block && (tl.lanes & (tl.lanes - 1)) == 0);
    CHECK(tl.lanes * 4 * qv2::kRowRegVecs >= tl.inner && tl.rows * tl.lanes <= block);
    CHECK(wide == (tl.inner > qv2::kBlockRows * 4 * qv2::kRowRegVecs));
    CHECK(static_cast<int64_t>(tl.rows) * tl.inner == tl.len);
    CHECK((reinterpret_cast<uintptr_t>(tl.x) & 15u) == 0);
    CHECK(tl.q == nullptr || (reinterpret_cast<uintptr_t>(tl.q) & 15u) == 0);
    CHECK(tl.c == nullptr || (reinterpret_cast<uintptr_t>(tl.c) & 3u) == 0);
    mark(tl, true, true);
  }
  int64_t total_s = 0, total_e = 0;
  for (const Segment& sg : p->segments) { total_s += sg.snp; total_e += sg.enp; }
  for (int64_t i = 0; i < total_s; ++i) CHECK(hits_s[i] == 1);
  for (int64_t i = 0; i < total_e; ++i) CHECK(hits_e[i] == 1);
  CHECK(static_cast<size_t>(total_s) * sizeof(qv2::StatPartial) <= ws);
  CHECK(static_cast<size_t>(total_e) * sizeof(qv2::ErrPartial5) <= ws);

  // pair pass: slots in tensor order; fused pair ranges = the tensor's quantize partials
  int64_t pp = 0;
  for (int32_t t = 0; t < nt; ++t) {
    const qv2::PairTensor& pt = p->pair_tensors[t];
    if (pt.n) { CHECK(pt.part0 == pp); pp += pt.nparts; }
    const qv2::PairTensor& ft = p->fused_pair_tensors[t];
    if (ft.n) {
      int64_t lo = std::numeric_limits<int64_t>::max(), cnt = 0;
      for (int32_t k = 0; k < p->info[t].nseg; ++k) {
        const Segment& sg = p->segments[p->info[t].seg0 + k];
        lo = std::min<int64_t>(lo, sg.ep0);
        cnt += sg.enp;
      }
      CHECK(ft.part0 == lo && ft.nparts == cnt);
    }
  }
  CHECK(static_cast<int64_t>(pair_tiles.size()) == pp);
  CHECK(static_cast<size_t>(pp) * sizeof(qv2::ErrPartial) <= ws);
  for (size_t i = 0; i < pair_tiles.size(); ++i) CHECK(pair_tiles[i].part0 == static_cast<int32_t>(i));

  // fold lists
  std::vector<int32_t> bs, be, bp, bf;
  for (int64_t i = 0; i < nseg; ++i) {
    if (p->segments[i].snp > qv2::kFoldWaveMax) bs.push_back(static_cast<int32_t>(i));
    if (p->segments[i].enp > qv2::kFoldWaveMax) be.push_back(static_cast<int32_t>(i));
  }
  for (int32_t t = 0; t < nt; ++t) {
    if (p->pair_tensors[t].nparts > qv2::kFoldWaveMax) bp.push_back(t);
    if (p->fused_pair_tensors[t].nparts > qv2::kFoldWaveMax) bf.push_back(t);
  }
  CHECK(bs == p->big_stat_segments && be == p->big_err_segments);
  CHECK(bp == p->big_pair_tensors && bf == p->big_fused_pair_tensors);

  // histogram chunks
  {
    std::vector<char> seen(p->hist_tiles.size(), 0);
    for (const Tile& tl : p->hist_tiles) {
      CHECK(tl.part0 >= 0 && tl.part0 < static_cast<int32_t>(seen.size()) && !seen[tl.part0]);
      seen[tl.part0] = 1;
    }
    for (size_t i = 1; i < p->hist_tiles.size(); ++i) CHECK(p->hist_tiles[i - 1].len >= p->hist_tiles[i].len);
  }
  for (int32_t t = 0; t < nt; ++t) {
    const qv2::HistTensor& ht = p->hist_tensors[t];
    CHECK(ht.seg0 == p->info[t].seg0 && ht.nseg == p->info[t].nseg && ht.nchunks >= 1);
    int32_t mine = 0;                      // the tensor's chunks own exactly its range of partial slots
    for (const Tile& tl : p->hist_tiles)
      if (tl.tensor == t) { CHECK(tl.part0 >= ht.chunk0 && tl.part0 < ht.chunk0 + ht.nchunks); ++mine; }
    CHECK(mine == ht.nchunks);
  }
  CHECK(qv2_histogram_workspace_bytes(p, 0) == 0 && qv2_histogram_workspace_bytes(p, qv2::kHistMaxBins + 1) == 0);
  CHECK(qv2_histogram_workspace_bytes(p, 2048) >= p->hist_tiles.size() * 2048 * sizeof(uint32_t));

  // finalize over made-up records of the right shape
  std::vector<qv2_qparams> params(nseg);
  std::vector<qv2_sums> sums(nseg);
  std::mt19937_64 g(nseg * 7919 + nt);
  std::uniform_real_distribution<double> u(0.1, 10.0);
  for (int64_t i = 0; i < nseg; ++i) {
    params[i] = qv2_qparams{-1.0f, 2.0f, 0.01f, 100.0f, 3, 0};
    const double n = static_cast<double>(p->segments[i].n);
    sums[i] = qv2_sums{0.5 * n, u(g) * n, 1e-4 * u(g) * n, p->segments[i].n};
  }
  std::vector<qv2_metrics> met(nt);
  CHECK(qv2_finalize(p, params.data(), sums.data(), met.data()) == QV2_OK);
  for (int32_t t = 0; t < nt; ++t) {
    CHECK(std::isfinite(met[t].mse) && met[t].mse > 0 && std::isfinite(met[t].sqnr_db));
    CHECK(met[t].min == -1.0f && met[t].max == 2.0f && met[t].absmax == 2.0f);
    CHECK(std::fabs(met[t].mean - 0.5) < 1e-12);
  }
  sums[0].sum_e2 = std::numeric_limits<double>::quiet_NaN();
  CHECK(qv2_finalize(p, params.data(), sums.data(), met.data()) == QV2_ERR_NONFINITE);
  CHECK(qv2_finalize(nullptr, params.data(), sums.data(), met.data()) == QV2_ERR_NULL);

  delete p;      // host tables only: nothing was uploaded, so no device memory to release
}

void plans() {
  std::mt19937_64 g(12345);
  auto pick = [&](int64_t lo, int64_t hi) { return lo + static_cast<int64_t>(g() % static_cast<uint64_t>(hi - lo + 1)); };
  // hand-made corner tables
  const int64_t lens[] = {1, 2, 3, 4, 5, 2047, 2048, 2049, 8191, 8192, 8193, 32767, 32768, 32769, 65536 + 5,
                          262144 * 129 + 7, (int64_t{1} << 31) + 4099};
  {
    std::vector<qv2_tensor> rows;
    uint64_t at = 0;
    for (int64_t n : lens)
      for (int scheme : {QV2_ASYM_TENSOR, QV2_SYM_TENSOR}) {
        qv2_tensor r{};
        r.x = fake_f32(at + 1); r.numel = n; r.channels = 1; r.scheme = scheme;
        r.qrun = (n % 2) ? fake_f32(at + (int64_t{1} << 33)) : nullptr;
        r.codes = (n % 3) ? fake_i8(at + 3) : nullptr;
        r.layer = static_cast<int32_t>(rows.size());
        rows.push_back(r);
        at += static_cast<uint64_t>(n) + 16;
      }
    check_plan(rows);
  }
  {
    const int64_t shapes[][2] = {{7, 1}, {5000, 1}, {33, 3}, {960, 9}, {3000, 3}, {1100, 9}, {64, 27}, {10, 64},
                                 {10, 65}, {37, 576}, {3, 8191}, {5, 8192}, {3, 8193}, {4, 20001}, {1, 17},
                                 {2, 40000}, {3, 70001}, {4096, 25088}, {1, 300000000}, {2049, 1024}, {512, 4608}};
    std::vector<qv2_tensor> rows;
    uint64_t at = 0;
    for (const auto& sh : shapes) {
      qv2_tensor r{};
      r.x = fake_f32(at + 2); r.numel = sh[0] * sh[1]; r.channels = static_cast<int32_t>(sh[0]);
      r.scheme = QV2_SYM_CHANNEL;
      r.qrun = (rows.size() % 2) ? fake_f32(at + (int64_t{1} << 34) + 1) : nullptr;
      r.codes = fake_i8(at + 1);
      rows.push_back(r);
      at += static_cast<uint64_t>(r.numel) + 8;
    }
    check_plan(rows);
  }
  // random tables
  for (int rep = 0; rep < 60; ++rep) {
    std::vector<qv2_tensor> rows;
    uint64_t at = 0;
    const int nt = static_cast<int>(pick(1, 40));
    for (int t = 0; t < nt; ++t) {
      qv2_tensor r{};
      const int kind = static_cast<int>(pick(0, 3));
      if (kind == 0) {                       // per-channel, short rows
        r.channels = static_cast<int32_t>(pick(1, 3000)); r.numel = r.channels * pick(1, 700);
        r.scheme = QV2_SYM_CHANNEL;
      } else if (kind == 1) {                // per-channel, long rows
        r.channels = static_cast<int32_t>(pick(1, 40)); r.numel = r.channels * pick(4000, 300000);
        r.scheme = QV2_SYM_CHANNEL;
      } else {                               // per-tensor
        r.channels = 1; r.numel = pick(1, 1) * pick(1, kind == 2 ? 100000 : 30000000);
        r.scheme = (g() & 1) ? QV2_ASYM_TENSOR : QV2_SYM_TENSOR;
      }
      r.x = fake_f32(at + pick(0, 3));
      r.qrun = (g() & 1) ? fake_f32(at + (int64_t{1} << 35) + pick(0, 3)) : nullptr;
      r.codes = (g() % 4) ? fake_i8(at + pick(0, 3)) : nullptr;
      r.kind = static_cast<int32_t>(g() & 1); r.layer = t;
      rows.push_back(r);
      at += static_cast<uint64_t>(r.numel) + 16;
    }
    check_plan(rows);
  }
  // rejected tables
  qv2_plan* p = nullptr;
  qv2_tensor r{};
  r.x = fake_f32(0); r.numel = 10; r.channels = 1; r.scheme = QV2_ASYM_TENSOR;
  CHECK(qv2_plan_create(nullptr, 1, &p) == QV2_ERR_NULL);
  CHECK(qv2_plan_create(&r, 0, &p) == QV2_ERR_SHAPE);
  CHECK(qv2_plan_create(&r, 1, nullptr) == QV2_ERR_NULL);
  qv2_tensor bad = r; bad.numel = 0;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE);
  bad = r; bad.scheme = 7;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SCHEME);
  bad = r; bad.scheme = QV2_SYM_CHANNEL; bad.channels = 3;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE);
  bad = r; bad.channels = 2;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE);
  bad = r; bad.x = reinterpret_cast<const float*>(0x1002);
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_ALIGN);
  bad = r; bad.x = nullptr;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_NULL);
  bad = r; bad.numel = (int64_t{1} << 36) + 1;                  // beyond the largest tensor a plan takes
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE);
  bad.scheme = QV2_SYM_CHANNEL; bad.channels = 1; bad.codes = reinterpret_cast<int8_t*>(0x2000);
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE);
  // a sweep is one launch of at most 2^32 - 1 threads: 2^24 quantize tiles of 256 threads are one
  // too many, the same tensor without a code buffer (long read-only tiles) fits
  bad = r; bad.numel = int64_t{1} << 35; bad.codes = reinterpret_cast<int8_t*>(0x2000);
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_ERR_SHAPE && p == nullptr);
  bad.numel -= qv2::kDefaultQuantTile;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_OK && p != nullptr);
  CHECK(qv2_plan_num_quant_tiles(p) == (int64_t{1} << 24) - 1);
  delete p; p = nullptr;
  bad.numel = int64_t{1} << 35; bad.codes = nullptr;
  CHECK(qv2_plan_create(&bad, 1, &p) == QV2_OK && p != nullptr);
  delete p; p = nullptr;
}

void ranking() {
  std::mt19937_64 g(777);
  std::normal_distribution<double> nd(30.0, 8.0);
  std::uniform_real_distribution<double> u(0.0, 1.0);
  const double inf = std::numeric_limits<double>::infinity(), nan = std::numeric_limits<double>::quiet_NaN();
  for (int rep = 0; rep < 400; ++rep) {
    const int n = 1 + static_cast<int>(g() % 160);
    std::vector<double> ws(n), as(n), wm(n), am(n), pos(n);
    for (int i = 0; i < n; ++i) {
      ws[i] = (g() % 23 == 0) ? inf : std::round(nd(g) * 4) / 4;      // ties on purpose
      as[i] = std::round(nd(g) * 4) / 4;
      wm[i] = u(g) * ((g() % 17 == 0) ? 100.0 : 1.0);
      am[i] = u(g) * ((g() % 13 == 0) ? 50.0 : 1.0);
      pos[i] = (i ? pos[i - 1] : 0.0) + 1 + static_cast<double>(g() % 3);
    }
    qv2_rank_config cfg;
    qv2_rank_config_default(&cfg);
    cfg.mse_source = static_cast<int32_t>(g() % 3);
    std::vector<int32_t> order(n, -1);
    std::vector<double> score(n);
    const bool with_a = g() % 4 != 0;
    if (!with_a) cfg.mse_source = 1;         // no activation series: only the weight MSE can feed the rule
    std::vector<int32_t> ipos(n);
    for (int i = 0; i < n; ++i) ipos[i] = static_cast<int32_t>(pos[i]);
    CHECK(qv2_rank(ws.data(), with_a ? as.data() : nullptr, wm.data(), with_a ? am.data() : nullptr,
                   (g() & 1) ? ipos.data() : nullptr, n, &cfg, order.data(), (g() & 1) ? score.data() : nullptr) == QV2_OK);
    std::vector<int> seen(n, 0);
    for (int i = 0; i < n; ++i) { CHECK(order[i] >= 0 && order[i] < n); ++seen[order[i]]; }
    for (int i = 0; i < n; ++i) CHECK(seen[i] == 1);

    // the steps after the ranking
    std::vector<double> macs(n);
    for (int i = 0; i < n; ++i) macs[i] = 1e6 * (1 + static_cast<double>(g() % 50));
    std::vector<uint8_t> keep(n);
    int32_t kept = -1;
    double pct = -1.0;
    const double target = 20.0 + 10.0 * static_cast<double>(g() % 6);
    CHECK(qv2_bops_select(order.data(), macs.data(), n, target, keep.data(), &kept, &pct) == QV2_OK);
    CHECK(kept >= 0 && kept <= n && pct <= 75.0 + 1e-9);
    int cnt = 0;
    for (int i = 0; i < n; ++i) cnt += keep[i] != 0;
    CHECK(cnt == kept);
    double pct2 = 0.0;
    CHECK(qv2_bops_reduction_pct(macs.data(), keep.data(), n, &pct2) == QV2_OK);
    CHECK(std::fabs(pct - pct2) < 1e-9);
    std::vector<int32_t> grp(n), out(n);
    for (int i = 0; i < n; ++i) grp[i] = (g() % 3 == 0) ? -1 : static_cast<int32_t>(g() % 9);
    CHECK(qv2_regroup_for_fusion(order.data(), grp.data(), n, out.data()) == QV2_OK);
    std::fill(seen.begin(), seen.end(), 0);
    for (int i = 0; i < n; ++i) { CHECK(out[i] >= 0 && out[i] < n); ++seen[out[i]]; }
    for (int i = 0; i < n; ++i) CHECK(seen[i] == 1);
    for (int kind = 0; kind < 2; ++kind) {
      CHECK(qv2_baseline_order(kind, ws.data(), n, out.data()) == QV2_OK);
      std::fill(seen.begin(), seen.end(), 0);
      for (int i = 0; i < n; ++i) { CHECK(out[i] >= 0 && out[i] < n); ++seen[out[i]]; }
      for (int i = 0; i < n; ++i) CHECK(seen[i] == 1);
    }
  }
  // hostile inputs come back as statuses
  double a[3] = {1.0, nan, 3.0}, b[3] = {1.0, 2.0, 3.0};
  int32_t o[3];
  CHECK(qv2_rank(a, b, b, b, nullptr, 3, nullptr, o, nullptr) == QV2_ERR_NONFINITE);
  CHECK(qv2_rank(b, b, b, b, nullptr, 0, nullptr, o, nullptr) == QV2_ERR_SHAPE);
  CHECK(qv2_rank(nullptr, nullptr, b, b, nullptr, 3, nullptr, o, nullptr) == QV2_ERR_NULL);
  CHECK(qv2_rank(nullptr, b, b, b, nullptr, 3, nullptr, o, nullptr) == QV2_OK);       // one series may be absent
  int32_t badpos[3] = {0, 2, 2};
  CHECK(qv2_rank(b, b, b, b, badpos, 3, nullptr, o, nullptr) == QV2_ERR_SHAPE);
  int32_t dup[3] = {0, 1, 1};
  uint8_t k3[3];
  int32_t kept;
  CHECK(qv2_bops_select(dup, b, 3, 50.0, k3, &kept, nullptr) == QV2_ERR_SHAPE);
  CHECK(qv2_regroup_for_fusion(dup, dup, 3, o) == QV2_ERR_SHAPE);
}

void rank_from_records() {
  std::mt19937_64 g(4242);
  std::uniform_real_distribution<double> u(0.5, 2.0);
  for (int rep = 0; rep < 50; ++rep) {
    const int n = 1 + static_cast<int>(g() % 60);
    std::vector<qv2_tensor> rows;
    for (int l = 0; l < n; ++l)
      for (int kind = 0; kind < 2; ++kind) {
        qv2_tensor r{};
        r.x = fake_f32(rows.size() * 4096); r.numel = 100 + l; r.channels = 1; r.scheme = QV2_ASYM_TENSOR;
        r.qrun = kind ? fake_f32((int64_t{1} << 30) + rows.size() * 4096) : nullptr;
        r.kind = kind; r.layer = l;
        rows.push_back(r);
      }
    std::shuffle(rows.begin(), rows.end(), g);
    qv2_plan* p = nullptr;
    CHECK(qv2_plan_create(rows.data(), static_cast<int32_t>(rows.size()), &p) == QV2_OK);
    std::vector<qv2_tensor_sums> ts(rows.size());
    std::vector<qv2_pair_sums> ps(rows.size());
    for (size_t t = 0; t < rows.size(); ++t) {
      const double nn = static_cast<double>(rows[t].numel);
      ts[t] = qv2_tensor_sums{0.0, u(g) * nn, 1e-4 * u(g) * nn, rows[t].numel, -1.0f, 1.0f, {0, 0}};
      ps[t] = rows[t].qrun ? qv2_pair_sums{u(g) * nn, 1e-3 * u(g) * nn, rows[t].numel, 0} : qv2_pair_sums{0, 0, 0, 0};
    }
    std::vector<int32_t> order(n, -1);
    std::vector<double> score(n);
    CHECK(qv2_rank_tensors(p, ts.data(), ps.data(), nullptr, n, nullptr, order.data(), score.data()) == QV2_OK);
    std::vector<int> seen(n, 0);
    for (int i = 0; i < n; ++i) { CHECK(order[i] >= 0 && order[i] < n); ++seen[order[i]]; }
    for (int i = 0; i < n; ++i) CHECK(seen[i] == 1);
    CHECK(qv2_rank_tensors(p, ts.data(), nullptr, nullptr, n, nullptr, order.data(), nullptr) == QV2_ERR_NULL);
    CHECK(qv2_rank_tensors(p, ts.data(), ps.data(), nullptr, n + 1, nullptr, order.data(), nullptr) == QV2_ERR_SHAPE);
    if (n > 1)
      CHECK(qv2_rank_tensors(p, ts.data(), ps.data(), nullptr, n - 1, nullptr, order.data(), nullptr) == QV2_ERR_SHAPE);
    CHECK(qv2_rank_tensors(nullptr, ts.data(), ps.data(), nullptr, n, nullptr, order.data(), nullptr) == QV2_ERR_NULL);
    delete p;
  }
}

void small_host_functions() {
  std::mt19937_64 g(99);
  for (int nb : {1, 2, 7, 256, 2048, 4096}) {
    std::vector<uint64_t> p(nb), q(nb);
    for (int i = 0; i < nb; ++i) { p[i] = g() % 1000; q[i] = g() % 1000; }
    p[0] += 1; q[0] += 1;
    double kl = -1.0;
    CHECK(qv2_kl_divergence(p.data(), q.data(), nb, 1e-6, &kl) == QV2_OK);
    CHECK(std::isfinite(kl) && kl >= -1e-12);
    CHECK(qv2_kl_divergence(p.data(), p.data(), nb, 0.0, &kl) == QV2_OK);
    CHECK(kl == 0.0);
  }
  double kl;
  uint64_t z[4] = {0, 0, 0, 0}, one[4] = {1, 0, 0, 0};
  CHECK(qv2_kl_divergence(z, one, 4, 0.0, &kl) != QV2_OK);              // empty histogram
  CHECK(qv2_kl_divergence(one, one, 0, 0.0, &kl) == QV2_ERR_SHAPE);
  CHECK(qv2_kl_divergence(one, one, 4, -1.0, &kl) != QV2_OK);

  qv2_pair_sums ps[3] = {{4.0, 1.0, 4, 0}, {4.0, 0.0, 4, 0}, {0.0, 0.0, 0, 0}};
  double mse[3], sq[3];
  CHECK(qv2_pair_finalize(ps, 3, mse, sq) == QV2_OK);
  CHECK(mse[0] == 0.25 && std::fabs(sq[0] - 10.0 * std::log10(4.0)) < 1e-12);
  CHECK(mse[1] == 0.0 && std::isinf(sq[1]) && sq[1] > 0);
  CHECK(mse[2] == 0.0 && std::isinf(sq[2]) && sq[2] > 0);          // a tensor without a partner

  qv2_tensor_sums ts[2] = {{2.0, 6.0, 0.5, 4, -1.0f, 2.0f, {0, 0}}, {0.0, 0.0, 0.0, 8, 0.0f, 0.0f, {0, 0}}};
  qv2_metrics m[2];
  CHECK(qv2_finalize_tensors(ts, 2, m) == QV2_OK);
  CHECK(m[0].mse == 0.125 && m[0].mean == 0.5 && m[0].var == 1.25 && m[0].absmax == 2.0f);
  CHECK(m[1].mse == 0.0 && std::isinf(m[1].sqnr_db));
  for (int s = 1; s >= -10; --s) CHECK(qv2_status_string(static_cast<qv2_status>(s)) != nullptr);
}

void config_file(const char* dir) {
  const std::string path = std::string(dir) + "/qv2_host_checks_config.csv";
  const uint8_t keep[4] = {1, 0, 0, 7};
  const char* names[4] = {"conv1", "layer1.0.conv1", "layer1.0.conv2", "fc"};
  CHECK(qv2_write_config(path.c_str(), keep, names, 4) == QV2_OK);
  std::FILE* f = std::fopen(path.c_str(), "r");
  CHECK(f != nullptr);
  char buf[256] = {};
  const size_t got = std::fread(buf, 1, sizeof buf - 1, f);
  std::fclose(f);
  CHECK(std::string(buf, got) == "layer,name,bits\n0,conv1,32\n1,layer1.0.conv1,8\n2,layer1.0.conv2,8\n3,fc,32\n");
  CHECK(qv2_write_config(path.c_str(), keep, nullptr, 2) == QV2_OK);
  const char* bad[2] = {"a", "b\nc"};
  CHECK(qv2_write_config(path.c_str(), keep, bad, 2) == QV2_ERR_SHAPE);
  const char* hole[2] = {"a", nullptr};
  CHECK(qv2_write_config(path.c_str(), keep, hole, 2) == QV2_ERR_NULL);
  CHECK(qv2_write_config((std::string(dir) + "/no/such/dir/x").c_str(), keep, nullptr, 2) == QV2_ERR_IO);
  std::remove(path.c_str());
}

}  // namespace

// the XCD-aware tile order of the sweeps is a permutation of the tile indices for any launch size
void tile_order() {
  for (int block : {1, 16, 256}) {
    for (int n : {1, 7, 8, 127, 128, 129, 2047, 2048, 2049, 4095, 4096, 12345, 82720, 1323517}) {
      std::vector<uint8_t> seen(static_cast<size_t>(n), 0);
      for (int k = 0; k < n; ++k) {
        const int t = qv2::xcd_blocked(k, n, block);
        CHECK(t >= 0 && t < n);
        CHECK(!seen[static_cast<size_t>(t)]);
        seen[static_cast<size_t>(t)] = 1;
      }
      // consecutive workgroups of one XCD (k, k + 8, ...) take neighbouring tiles inside a whole group
      if (n >= 16 * block && block > 1)
        CHECK(qv2::xcd_blocked(8, n, block) == qv2::xcd_blocked(0, n, block) + 1);
    }
  }
}

int main(int argc, char** argv) {
  config_file(argc > 1 ? argv[1] : "/tmp");
  plans();
  ranking();
  rank_from_records();
  small_host_functions();
  tile_order();
  std::printf("host checks ok\n");
  return 0;
}
