// Host side of the qv2 C ABI: the plan builder (layer table -> flat tile
// table), the fp64 finalize of Sec. 6.1 Eq. 6-7, and the sensitivity ranking of
// Sec. 6.4 Eq. 16 / Algorithm 2.  No GPU is needed by anything in this file.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

#include "qv2_internal.h"

using qv2::PairTensor;
using qv2::Run;
using qv2::Segment;
using qv2::StreamTable;
using qv2::TensorInfo;
using qv2::Tile;

namespace {

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Tile length from an environment variable (tuning sweeps), else the default.
int32_t tile_from_env(const char* name, int32_t dflt) {
  const char* e = std::getenv(name);
  if (!e || !*e) return dflt;
  long v = std::strtol(e, nullptr, 10);
  if (v < 256) v = 256;
  if (v > (1L << 22)) v = 1L << 22;
  return static_cast<int32_t>(v / 4 * 4);
}

// Appends the stream tiles of one tensor (nseg segments of `inner` elements, cut into tiles of T
// elements, partial slots from part0) to a table; returns the number of tiles added.
int64_t add_run(StreamTable& tab, const qv2_tensor& in, int32_t t, int64_t nseg, int64_t inner, int64_t T,
                int64_t seg0, int64_t part0) {
  const int64_t per_seg = (inner + T - 1) / T;
  Run r{};
  r.x = in.x; r.q = in.qrun; r.c = in.codes;
  r.inner = inner;
  r.tile0 = static_cast<int32_t>(tab.n_tiles);
  r.tiles_per_seg = static_cast<int32_t>(per_seg);
  r.seg0 = static_cast<int32_t>(seg0);
  r.part0 = static_cast<int32_t>(part0);
  r.tile_len = static_cast<int32_t>(T);
  r.tensor = t;
  r.tile_end = static_cast<int32_t>(tab.n_tiles + nseg * per_seg);
  tab.runs.push_back(r);
  tab.n_tiles += nseg * per_seg;
  return nseg * per_seg;
}

// The lookup table from blocks of 2^shift tile indices to runs.
void finish_table(StreamTable& tab) {
  tab.shift = 0;
  while ((tab.n_tiles >> tab.shift) + 1 > qv2::kCoarseMax) ++tab.shift;
  const int64_t n = (tab.n_tiles >> tab.shift) + 1;
  tab.coarse.assign(static_cast<size_t>(n), 0);
  size_t r = 0;
  for (int64_t b = 0; b < n; ++b) {
    const int64_t k = b << tab.shift;
    while (r + 1 < tab.runs.size() && tab.runs[r + 1].tile0 <= k) ++r;
    tab.coarse[static_cast<size_t>(b)] = static_cast<int32_t>(r);
  }
}

// How the rows of a per-channel tensor are handled: as stream tiles, staged in LDS, or held in
// registers (rows of whole 16-byte vectors on 16-byte boundaries, coded through whole dwords).
qv2::RowForm row_form(const qv2_tensor& in, int64_t inner) {
  if (in.scheme != QV2_SYM_CHANNEL) return qv2::kRowStream;
  const bool reg_ok = inner % 4 == 0 && inner >= qv2::kRowRegMinInner &&
                      (reinterpret_cast<uintptr_t>(in.x) & 15u) == 0 &&
                      (!in.qrun || (reinterpret_cast<uintptr_t>(in.qrun) & 15u) == 0) &&
                      (!in.codes || (reinterpret_cast<uintptr_t>(in.codes) & 3u) == 0);
  if (reg_ok && inner <= int64_t{qv2::kBlockRows} * 4 * qv2::kRowRegVecs) return qv2::kRowReg;
  if (reg_ok && inner <= qv2::kRowRegCap) return qv2::kRowRegWide;
  return inner <= qv2::kRowGroupCap ? qv2::kRowLds : qv2::kRowStream;
}

// A launch of n workgroups of `block` threads must stay within 2^32 - 1 threads in all.
bool launchable(int64_t n, int64_t block) { return n * block <= int64_t{0xFFFFFFFF}; }

// Runs a host entry point's body; an allocation failure inside it becomes a status.
template <class F>
qv2_status guarded(F&& body) {
  try {
    return body();
  } catch (...) {            // only allocations can throw in these bodies
    return QV2_ERR_NOMEM;
  }
}

}  // namespace

extern "C" {

static qv2_status plan_create(const qv2_tensor* h_tensors, int32_t n_tensors, qv2_plan* p);

qv2_status qv2_plan_create(const qv2_tensor* h_tensors, int32_t n_tensors, qv2_plan** out) {
  if (!h_tensors || !out) return QV2_ERR_NULL;
  *out = nullptr;
  if (n_tensors <= 0) return QV2_ERR_SHAPE;
  qv2_plan* p = new (std::nothrow) qv2_plan();
  if (!p) return QV2_ERR_NOMEM;
  // the tile tables grow with the input: a failed allocation must not leave as an exception
  const qv2_status st = guarded([&]() -> qv2_status { return plan_create(h_tensors, n_tensors, p); });
  if (st != QV2_OK) { delete p; return st; }
  *out = p;
  return QV2_OK;
}

static qv2_status plan_create(const qv2_tensor* h_tensors, int32_t n_tensors, qv2_plan* p) {
  const int64_t kMax = std::numeric_limits<int32_t>::max();

  // validate, and count the row-group partials: they are numbered first
  int64_t n_row_parts = 0, n_segments = 0;
  for (int32_t t = 0; t < n_tensors; ++t) {
    const qv2_tensor& in = h_tensors[t];
    if (!in.x) return QV2_ERR_NULL;
    if (in.numel <= 0 || in.numel > qv2::kMaxNumel) return QV2_ERR_SHAPE;
    if (in.scheme != QV2_ASYM_TENSOR && in.scheme != QV2_SYM_TENSOR && in.scheme != QV2_SYM_CHANNEL)
      return QV2_ERR_SCHEME;
    const bool per_channel = in.scheme == QV2_SYM_CHANNEL;
    if (per_channel ? (in.channels <= 0 || in.numel % in.channels != 0) : in.channels != 1)
      return QV2_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(in.x) & 3u) ||
        (in.qrun && (reinterpret_cast<uintptr_t>(in.qrun) & 3u))) return QV2_ERR_ALIGN;
    const int64_t nseg = per_channel ? in.channels : 1;
    n_segments += nseg;
    if (row_form(in, in.numel / nseg) != qv2::kRowStream) n_row_parts += nseg;
    if (n_segments > kMax) return QV2_ERR_SHAPE;
  }

  p->read_tile = tile_from_env("QV2_TILE_ELEMS", qv2::kDefaultReadTile);
  p->quant_tile = tile_from_env("QV2_QUANT_TILE_ELEMS", qv2::kDefaultQuantTile);
  const int64_t TR = p->read_tile, TQ = p->quant_tile;
  p->n_row_parts = static_cast<int32_t>(n_row_parts);

  int64_t row_part = 0;                      // next row-group partial (same in both numberings)
  int64_t sp = n_row_parts, ep = n_row_parts, pp = 0;   // next stream partial: stats / quantize / pair
  qv2_status err = QV2_OK;

  auto make_tile = [](const qv2_tensor& in, int32_t t, int64_t off, int64_t len) {
    Tile tl{};
    tl.x = in.x + off;
    tl.q = in.qrun ? in.qrun + off : nullptr;
    tl.c = in.codes ? in.codes + off : nullptr;
    tl.len = static_cast<int32_t>(len);
    tl.tensor = t;
    return tl;
  };

  for (int32_t t = 0; t < n_tensors; ++t) {
    const qv2_tensor& in = h_tensors[t];
    const bool per_channel = in.scheme == QV2_SYM_CHANNEL;
    const int64_t nseg = per_channel ? in.channels : 1;
    const int64_t inner = in.numel / nseg;
    const int64_t seg0 = static_cast<int64_t>(p->segments.size());
    p->info.push_back(TensorInfo{in.numel, static_cast<int32_t>(seg0), static_cast<int32_t>(nseg), in.kind,
                                 in.layer, in.qrun != nullptr});

    PairTensor ft{};                         // this tensor's partials in the quantize numbering
    PairTensor st{};                         // ... in the calibration numbering (stream tiles only)
    const qv2::RowForm form = row_form(in, inner);
    if (form != qv2::kRowStream) {
      // whole rows per tile; every row is its own segment with one partial
      ft.part0 = static_cast<int32_t>(row_part); ft.nparts = static_cast<int32_t>(nseg);
      p->n_single_read += in.numel;
      // rows of whole 16-byte vectors on 16-byte boundaries are held in registers: `lanes`
      // lanes per row (each at most kRowRegVecs vectors), one round of rows per workgroup
      const bool reg_form = form != qv2::kRowLds;
      int64_t lanes = 0, rpt = 0;
      if (reg_form) {
        lanes = qv2::kRowRegMinLanes;
        while (lanes * 4 * qv2::kRowRegVecs < inner) lanes <<= 1;
        rpt = (form == qv2::kRowRegWide ? qv2::kBlockRowsWide : qv2::kBlockRows) / lanes;
      } else {
        // otherwise staged in LDS.  Rows per tile: what fits the LDS copy, but no more than a
        // few rounds of the row kernels (a round = one row per lane group of every wavefront),
        // so that a tile of very short rows does not become the longest-running workgroup
        int64_t group = 1;
        while (group < inner && group < 64) group <<= 1;
        const int64_t per_round = (qv2::kBlockRows / 64) * (64 / group);
        rpt = std::min<int64_t>({qv2::kRowGroupMaxRows, qv2::kRowGroupCap / inner,
                                 qv2::kRowGroupRounds * per_round});
      }
      if (in.qrun) p->rows_have_pair = true;
      for (int64_t r0 = 0; r0 < nseg; r0 += rpt) {
        const int64_t rows = std::min(rpt, nseg - r0);
        Tile tl = make_tile(in, t, r0 * inner, rows * inner);
        tl.part0 = static_cast<int32_t>(row_part + r0); tl.rows = static_cast<int32_t>(rows);
        tl.seg0 = static_cast<int32_t>(seg0 + r0); tl.inner = static_cast<int32_t>(inner);
        tl.lanes = static_cast<int32_t>(lanes);
        (form == qv2::kRowRegWide ? p->wide_tiles : reg_form ? p->reg_tiles : p->row_tiles).push_back(tl);
      }
      for (int64_t r = 0; r < nseg; ++r) {
        Segment s{};
        s.n = inner; s.scheme = in.scheme; s.tensor = t;
        s.sp0 = s.ep0 = static_cast<int32_t>(row_part + r); s.snp = s.enp = 1;
        p->segments.push_back(s);
      }
      p->row_tensors.push_back(t);
      row_part += nseg;
    } else {
      // without a code buffer the quantize sweep stores nothing: long tiles, as for a read-only pass
      const int64_t TQt = in.codes ? TQ : TR;
      const int64_t n_read = (inner + TR - 1) / TR, n_quant = (inner + TQt - 1) / TQt;
      if (sp + nseg * n_read > kMax || ep + nseg * n_quant > kMax) { err = QV2_ERR_SHAPE; break; }
      ft.part0 = static_cast<int32_t>(ep); ft.nparts = static_cast<int32_t>(nseg * n_quant);
      st.part0 = static_cast<int32_t>(sp); st.nparts = static_cast<int32_t>(nseg * n_read);
      if (in.qrun) st.n = in.numel;
      // the tensor's tiles: segment after segment, each segment's tiles in element order, one
      // partial slot per tile in that same order
      add_run(p->read_tiles, in, t, nseg, inner, TR, seg0, sp);
      add_run(in.codes ? p->quant_tiles : p->quant_ro_tiles, in, t, nseg, inner, TQt, seg0, ep);
      if (nseg > 1) p->late_tensors.push_back(t);
      for (int64_t s = 0; s < nseg; ++s) {
        Segment sg{};
        sg.n = inner; sg.scheme = in.scheme; sg.tensor = t;
        sg.sp0 = static_cast<int32_t>(sp); sg.snp = static_cast<int32_t>(n_read);
        sg.ep0 = static_cast<int32_t>(ep); sg.enp = static_cast<int32_t>(n_quant);
        p->segments.push_back(sg);
        sp += n_read; ep += n_quant;
      }
    }
    if (in.qrun) ft.n = in.numel; else ft = PairTensor{};
    p->fused_pair_tensors.push_back(ft);
    if (!in.qrun) st = PairTensor{};
    p->stat_pair_tensors.push_back(st);

    PairTensor pt{};
    if (in.qrun) {
      const int64_t nt = (in.numel + TR - 1) / TR;
      if (pp + nt > kMax) { err = QV2_ERR_SHAPE; break; }
      pt.n = in.numel; pt.part0 = static_cast<int32_t>(pp); pt.nparts = static_cast<int32_t>(nt);
      pp += add_run(p->pair_tiles, in, t, 1, in.numel, TR, seg0, pp);     // the whole tensor as one range
    }
    p->pair_tensors.push_back(pt);
  }
  if (err != QV2_OK) return err;
  // every sweep is one launch: its tile count times its workgroup size has to fit a launch
  if (!launchable(p->read_tiles.n_tiles, qv2::kBlockRead) || !launchable(p->pair_tiles.n_tiles, qv2::kBlockRead) ||
      !launchable(p->quant_ro_tiles.n_tiles, qv2::kBlockRead) ||
      !launchable(p->quant_tiles.n_tiles, qv2::kBlockQuant) ||
      !launchable(static_cast<int64_t>(std::max(p->row_tiles.size(), p->reg_tiles.size())), qv2::kBlockRows) ||
      !launchable(static_cast<int64_t>(p->wide_tiles.size()), qv2::kBlockRowsWide))
    return QV2_ERR_SHAPE;
  finish_table(p->read_tiles); finish_table(p->quant_tiles);
  finish_table(p->quant_ro_tiles); finish_table(p->pair_tiles);

  // histogram pass: about kHistChunks long chunks over all tensors
  {
    int64_t total = 0;
    for (int32_t t = 0; t < n_tensors; ++t) total += h_tensors[t].numel;
    int64_t chunk = (total + qv2::kHistChunks - 1) / qv2::kHistChunks;
    chunk = std::max<int64_t>(qv2::kHistMinChunk, (chunk + 4095) / 4096 * 4096);
    chunk = std::min<int64_t>(chunk, int64_t{1} << 30);
    for (int32_t t = 0; t < n_tensors; ++t) {
      const qv2_tensor& in = h_tensors[t];
      const int64_t nc = (in.numel + chunk - 1) / chunk;
      qv2::HistTensor ht{static_cast<int32_t>(p->hist_tiles.size()), static_cast<int32_t>(nc),
                         p->info[t].seg0, p->info[t].nseg};
      if (static_cast<int64_t>(p->hist_tiles.size()) + nc > kMax) return QV2_ERR_SHAPE;
      for (int64_t k = 0; k < nc; ++k) {
        Tile tl = make_tile(in, t, k * chunk, std::min<int64_t>(chunk, in.numel - k * chunk));
        tl.part0 = static_cast<int32_t>(p->hist_tiles.size());
        p->hist_tiles.push_back(tl);
      }
      p->hist_tensors.push_back(ht);
    }
  }

  // launch order: longest chunks first, so the last workgroups to start are the short
  // remainders (a chunk's partial slot is its part0, not its place in this table)
  std::stable_sort(p->hist_tiles.begin(), p->hist_tiles.end(),
                   [](const Tile& a, const Tile& b) { return a.len > b.len; });

  for (size_t i = 0; i < p->segments.size(); ++i) {
    if (p->segments[i].snp > qv2::kFoldWaveMax) p->big_stat_segments.push_back(static_cast<int32_t>(i));
    if (p->segments[i].enp > qv2::kFoldWaveMax) p->big_err_segments.push_back(static_cast<int32_t>(i));
  }
  for (size_t i = 0; i < p->pair_tensors.size(); ++i) {
    if (p->pair_tensors[i].nparts > qv2::kFoldWaveMax) p->big_pair_tensors.push_back(static_cast<int32_t>(i));
    if (p->fused_pair_tensors[i].nparts > qv2::kFoldWaveMax)
      p->big_fused_pair_tensors.push_back(static_cast<int32_t>(i));
    if (p->stat_pair_tensors[i].nparts > qv2::kFoldWaveMax)
      p->big_stat_pair_tensors.push_back(static_cast<int32_t>(i));
  }
  const size_t need = std::max({static_cast<size_t>(sp) * sizeof(qv2::StatPairCosPartial),
                                static_cast<size_t>(ep) * sizeof(qv2::ErrPartial5),
                                static_cast<size_t>(pp) * sizeof(qv2::ErrPartial)});
  p->workspace_bytes = std::max<size_t>(256, round_up(need, 256));
  return QV2_OK;
}

int32_t qv2_plan_num_tensors(const qv2_plan* plan) {
  return plan ? static_cast<int32_t>(plan->info.size()) : 0;
}
int64_t qv2_plan_num_segments(const qv2_plan* plan) {
  return plan ? static_cast<int64_t>(plan->segments.size()) : 0;
}
int64_t qv2_plan_segment_begin(const qv2_plan* plan, int32_t t) {
  if (!plan || t < 0 || t >= static_cast<int32_t>(plan->info.size())) return -1;
  return plan->info[t].seg0;
}
int64_t qv2_plan_num_tiles(const qv2_plan* plan) {
  return plan ? plan->read_tiles.n_tiles + static_cast<int64_t>(plan->row_tiles.size() + plan->reg_tiles.size() +
                                                                plan->wide_tiles.size()) : 0;
}
int64_t qv2_plan_num_quant_tiles(const qv2_plan* plan) {
  return plan ? plan->quant_tiles.n_tiles + plan->quant_ro_tiles.n_tiles +
                    static_cast<int64_t>(plan->row_tiles.size() + plan->reg_tiles.size() + plan->wide_tiles.size()) : 0;
}
int64_t qv2_plan_num_pair_tiles(const qv2_plan* plan) {
  return plan ? plan->pair_tiles.n_tiles : 0;
}
int64_t qv2_plan_num_single_read_elements(const qv2_plan* plan) { return plan ? plan->n_single_read : 0; }
size_t qv2_workspace_bytes(const qv2_plan* plan) { return plan ? plan->workspace_bytes : 0; }

size_t qv2_histogram_workspace_bytes(const qv2_plan* plan, int32_t nbins) {
  if (!plan || nbins < 2 || nbins > qv2::kHistMaxBins) return 0;
  // per-tensor range records, then two partial histograms (x, qrun) per chunk
  const size_t ranges = round_up(plan->info.size() * 2 * sizeof(float), 256);
  return ranges + round_up(plan->hist_tiles.size() * 2 * static_cast<size_t>(nbins) * sizeof(uint32_t), 256);
}

// ---------------------------------------------------------------------------
// Sec. 6.1 Eq. 6-7 and the tensor statistics, fp64.
// ---------------------------------------------------------------------------
static double sqnr_db_of(double signal, double noise) {
  if (noise == 0.0) return std::numeric_limits<double>::infinity();
  return 10.0 * std::log10(signal / noise);
}

qv2_status qv2_finalize(const qv2_plan* plan, const qv2_qparams* h_params,
                        const qv2_sums* h_sums, qv2_metrics* h_out) {
  if (!plan || !h_params || !h_sums || !h_out) return QV2_ERR_NULL;
  bool finite = true;
  for (size_t t = 0; t < plan->info.size(); ++t) {
    const TensorInfo& d = plan->info[t];
    double sx = 0.0, sx2 = 0.0, se2 = 0.0;
    float mn = std::numeric_limits<float>::infinity(), mx = -mn;
    for (int32_t s = d.seg0; s < d.seg0 + d.nseg; ++s) {
      sx += h_sums[s].sum_x; sx2 += h_sums[s].sum_x2; se2 += h_sums[s].sum_e2;
      mn = std::min(mn, h_params[s].min); mx = std::max(mx, h_params[s].max);
    }
    finite = finite && std::isfinite(sx) && std::isfinite(sx2) && std::isfinite(se2);
    const double n = static_cast<double>(d.numel);
    qv2_metrics m{};
    m.mse = se2 / n;
    m.sqnr_db = sqnr_db_of(sx2, se2);
    m.mean = sx / n;
    m.var = std::max(0.0, sx2 / n - m.mean * m.mean);
    m.min = mn; m.max = mx; m.absmax = std::max(std::fabs(mn), std::fabs(mx));
    h_out[t] = m;
  }
  return finite ? QV2_OK : QV2_ERR_NONFINITE;
}

qv2_status qv2_finalize_tensors(const qv2_tensor_sums* h, int32_t n_tensors, qv2_metrics* h_out) {
  if (!h || !h_out) return QV2_ERR_NULL;
  if (n_tensors < 0) return QV2_ERR_SHAPE;
  bool finite = true;
  for (int32_t t = 0; t < n_tensors; ++t) {
    finite = finite && std::isfinite(h[t].sum_x) && std::isfinite(h[t].sum_x2) && std::isfinite(h[t].sum_e2);
    const double n = static_cast<double>(h[t].n);
    qv2_metrics m{};
    m.mse = h[t].sum_e2 / n;
    m.sqnr_db = sqnr_db_of(h[t].sum_x2, h[t].sum_e2);
    m.mean = h[t].sum_x / n;
    m.var = std::max(0.0, h[t].sum_x2 / n - m.mean * m.mean);
    m.min = h[t].min; m.max = h[t].max;
    m.absmax = std::max(std::fabs(h[t].min), std::fabs(h[t].max));
    h_out[t] = m;
  }
  return finite ? QV2_OK : QV2_ERR_NONFINITE;
}

qv2_status qv2_pair_finalize(const qv2_pair_sums* h_pair, int32_t n, double* h_mse,
                             double* h_sqnr_db) {
  if (!h_pair || !h_mse || !h_sqnr_db) return QV2_ERR_NULL;
  if (n < 0) return QV2_ERR_SHAPE;
  bool finite = true;
  for (int32_t i = 0; i < n; ++i) {
    finite = finite && std::isfinite(h_pair[i].sum_ref2) && std::isfinite(h_pair[i].sum_d2);
    h_mse[i] = h_pair[i].n > 0 ? h_pair[i].sum_d2 / static_cast<double>(h_pair[i].n) : 0.0;
    h_sqnr_db[i] = sqnr_db_of(h_pair[i].sum_ref2, h_pair[i].sum_d2);
  }
  return finite ? QV2_OK : QV2_ERR_NONFINITE;
}

// Sec. 6.1 Eq. 9 between two histograms over the same bins, natural log, fp64.
qv2_status qv2_kl_divergence(const uint64_t* h_hist_p, const uint64_t* h_hist_q, int32_t nbins,
                             double eps, double* kl_out) {
  if (!h_hist_p || !h_hist_q || !kl_out) return QV2_ERR_NULL;
  if (nbins <= 0) return QV2_ERR_SHAPE;
  if (!(eps >= 0.0) || !std::isfinite(eps)) return QV2_ERR_NONFINITE;
  double tp = 0.0, tq = 0.0;
  for (int32_t i = 0; i < nbins; ++i) {
    tp += static_cast<double>(h_hist_p[i]);
    tq += static_cast<double>(h_hist_q[i]);
  }
  tp += eps * nbins; tq += eps * nbins;
  if (!(tp > 0.0) || !(tq > 0.0)) return QV2_ERR_SHAPE;
  double kl = 0.0;
  for (int32_t i = 0; i < nbins; ++i) {
    const double pa = (static_cast<double>(h_hist_p[i]) + eps) / tp;
    const double qa = (static_cast<double>(h_hist_q[i]) + eps) / tq;
    if (pa == 0.0) continue;
    if (qa == 0.0) { *kl_out = std::numeric_limits<double>::infinity(); return QV2_OK; }
    kl += pa * std::log(pa / qa);
  }
  *kl_out = kl;
  return QV2_OK;
}

// Sec. 6.1 Eq. 8 from the energies the quantize pass keeps: with d = a - b,
// sum b^2 = sum d^2 - sum a^2 + 2 sum a*b.
static double cosine_from(double saa, double sdd, double sab) {
  const double sbb = std::max(0.0, sdd - saa + 2.0 * sab);
  if (saa == 0.0 || sbb == 0.0) return saa == sbb ? 1.0 : 0.0;
  return sab / (std::sqrt(saa) * std::sqrt(sbb));
}

qv2_status qv2_cosine_finalize(const qv2_plan* plan, const qv2_sums* h_sums, const double* h_seg_xxhat,
                               const qv2_pair_sums* h_pair, const double* h_pair_xq,
                               double* h_cos_quant, double* h_cos_pair) {
  if (!plan || !h_sums || !h_seg_xxhat || !h_pair || !h_pair_xq || !h_cos_quant || !h_cos_pair)
    return QV2_ERR_NULL;
  bool finite = true;
  for (size_t t = 0; t < plan->info.size(); ++t) {
    const TensorInfo& d = plan->info[t];
    double sx2 = 0.0, se2 = 0.0, sxh = 0.0;
    for (int32_t s = d.seg0; s < d.seg0 + d.nseg; ++s) {
      sx2 += h_sums[s].sum_x2; se2 += h_sums[s].sum_e2; sxh += h_seg_xxhat[s];
    }
    finite = finite && std::isfinite(sx2) && std::isfinite(se2) && std::isfinite(sxh) &&
             std::isfinite(h_pair[t].sum_ref2) && std::isfinite(h_pair[t].sum_d2) &&
             std::isfinite(h_pair_xq[t]);
    h_cos_quant[t] = cosine_from(sx2, se2, sxh);
    h_cos_pair[t] = h_pair[t].n > 0 ? cosine_from(h_pair[t].sum_ref2, h_pair[t].sum_d2, h_pair_xq[t])
                                    : std::numeric_limits<double>::quiet_NaN();
  }
  return finite ? QV2_OK : QV2_ERR_NONFINITE;
}

// ---------------------------------------------------------------------------
// Sec. 6.4 Eq. 16 and Algorithm 2.
// ---------------------------------------------------------------------------
void qv2_rank_config_default(qv2_rank_config* cfg) {
  if (!cfg) return;
  cfg->alpha_w = 0.6; cfg->alpha_a = 0.4; cfg->mse_factor = 5.0; cfg->sqnr_cap_db = 200.0;
  cfg->mse_source = 0; cfg->_pad = 0;
}

// Eq. 16 on one series; returns false on NaN input.
static bool sqnr_delta_series(const double* sqnr, const int32_t* pos, int32_t n, double cap,
                              std::vector<double>& delta) {
  delta.assign(n, 0.0);
  if (!sqnr) return true;
  double prev = 0.0;
  for (int32_t i = 0; i < n; ++i) {
    if (std::isnan(sqnr[i])) return false;
    const double cur = std::max(-cap, std::min(cap, sqnr[i]));
    if (i > 0) {
      const double dl = pos ? static_cast<double>(pos[i] - pos[i - 1]) : 1.0;
      delta[i] = (cur - prev) / dl;
    }
    prev = cur;
  }
  return true;
}

qv2_status qv2_rank(const double* w_sqnr_db, const double* a_sqnr_db, const double* w_mse,
                    const double* a_mse, const int32_t* layer_pos, int32_t n_layers,
                    const qv2_rank_config* cfg, int32_t* order_out, double* score_out) {
  return guarded([&]() -> qv2_status {
    if (!order_out || (!w_sqnr_db && !a_sqnr_db)) return QV2_ERR_NULL;
    if (n_layers <= 0) return QV2_ERR_SHAPE;
    qv2_rank_config c;
    if (cfg) c = *cfg; else qv2_rank_config_default(&c);
    if (c.mse_source < 0 || c.mse_source > 2) return QV2_ERR_SHAPE;
    const double* src[2] = {nullptr, nullptr};
    int nsrc = 0;
    if (c.mse_source == 1 || c.mse_source == 2) src[nsrc++] = w_mse;
    if (c.mse_source == 0 || c.mse_source == 2) src[nsrc++] = a_mse;
    for (int k = 0; k < nsrc; ++k) if (!src[k]) return QV2_ERR_NULL;
    if (layer_pos)
      for (int32_t i = 1; i < n_layers; ++i)
        if (layer_pos[i] <= layer_pos[i - 1]) return QV2_ERR_SHAPE;

    const int32_t n = n_layers;
    std::vector<double> dw, da, score(n), key(n, 0.0);
    if (!sqnr_delta_series(w_sqnr_db, layer_pos, n, c.sqnr_cap_db, dw) ||
        !sqnr_delta_series(a_sqnr_db, layer_pos, n, c.sqnr_cap_db, da)) return QV2_ERR_NONFINITE;
    for (int32_t i = 0; i < n; ++i) score[i] = c.alpha_w * dw[i] + c.alpha_a * da[i];

    // outliers: MSE strictly above mse_factor x the arithmetic mean of its list
    std::vector<char> outlier(n, 0);
    for (int k = 0; k < nsrc; ++k) {
      const double* m = src[k];
      double total = 0.0;
      for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(m[i]) || m[i] < 0.0) return QV2_ERR_NONFINITE;
        total += m[i];
      }
      const double mean = total / static_cast<double>(n);
      for (int32_t i = 0; i < n; ++i) {
        if (m[i] > c.mse_factor * mean) outlier[i] = 1;
        // one list: order outliers by their MSE; two lists: by MSE relative to the list's mean
        const double kk = nsrc == 1 ? m[i] : (mean > 0.0 ? m[i] / mean : 0.0);
        key[i] = std::max(key[i], kk);
      }
    }

    std::vector<int32_t> front, rest;
    for (int32_t i = 0; i < n; ++i) (outlier[i] ? front : rest).push_back(i);
    std::stable_sort(front.begin(), front.end(),
                     [&](int32_t a, int32_t b) { return key[a] > key[b]; });
    std::stable_sort(rest.begin(), rest.end(),
                     [&](int32_t a, int32_t b) { return score[a] < score[b]; });
    int32_t w = 0;
    for (int32_t i : front) order_out[w++] = i;
    for (int32_t i : rest) order_out[w++] = i;
    if (score_out) std::memcpy(score_out, score.data(), sizeof(double) * n);
    return QV2_OK;
  });
}

// ---------------------------------------------------------------------------
// Sec. 7: compile-time baseline orders and the BOPs reduction rate (Eq. 17).
// ---------------------------------------------------------------------------
// Per-layer series from the per-tensor records of a plan, then qv2_rank.
qv2_status qv2_rank_tensors(const qv2_plan* plan, const qv2_tensor_sums* h_tensor_sums,
                            const qv2_pair_sums* h_pair_sums, const int32_t* layer_pos, int32_t n_layers,
                            const qv2_rank_config* cfg, int32_t* order_out, double* score_out) {
  return guarded([&]() -> qv2_status {
    if (!plan || !h_tensor_sums || !order_out) return QV2_ERR_NULL;
    if (n_layers <= 0) return QV2_ERR_SHAPE;
    const double nan = std::numeric_limits<double>::quiet_NaN();
    std::vector<double> w_sqnr(n_layers, nan), w_mse(n_layers, nan), a_sqnr(n_layers, nan), a_mse(n_layers, nan);
    int32_t n_w = 0, n_a = 0;
    for (size_t t = 0; t < plan->info.size(); ++t) {
      const TensorInfo& d = plan->info[t];
      if (d.layer < 0 || d.layer >= n_layers) return QV2_ERR_SHAPE;
      if (d.kind == 0) {                                       // weight: Eq. 6-7 against its dequantized form
        if (!std::isnan(w_mse[d.layer])) return QV2_ERR_SHAPE;  // two weights in one layer
        const qv2_tensor_sums& u = h_tensor_sums[t];
        if (u.n <= 0) return QV2_ERR_SHAPE;
        w_mse[d.layer] = u.sum_e2 / static_cast<double>(u.n);
        w_sqnr[d.layer] = sqnr_db_of(u.sum_x2, u.sum_e2);
        ++n_w;
      } else if (d.has_pair) {                                 // activation: fp32 run against quantized run
        if (!h_pair_sums) return QV2_ERR_NULL;
        if (!std::isnan(a_mse[d.layer])) return QV2_ERR_SHAPE;
        const qv2_pair_sums& u = h_pair_sums[t];
        if (u.n <= 0) return QV2_ERR_SHAPE;
        a_mse[d.layer] = u.sum_d2 / static_cast<double>(u.n);
        a_sqnr[d.layer] = sqnr_db_of(u.sum_ref2, u.sum_d2);
        ++n_a;
      }
    }
    // a series is used only when every layer has an entry in it
    if ((n_w != 0 && n_w != n_layers) || (n_a != 0 && n_a != n_layers) || (n_w == 0 && n_a == 0))
      return QV2_ERR_SHAPE;
    return qv2_rank(n_w ? w_sqnr.data() : nullptr, n_a ? a_sqnr.data() : nullptr, n_w ? w_mse.data() : nullptr,
                    n_a ? a_mse.data() : nullptr, layer_pos, n_layers, cfg, order_out, score_out);
  });
}

qv2_status qv2_baseline_order(int32_t kind, const double* w_sqnr_db, int32_t n_layers,
                              int32_t* order_out) {
  if (!order_out) return QV2_ERR_NULL;
  if (n_layers <= 0) return QV2_ERR_SHAPE;
  if (kind == QV2_ORDER_INORDER) {
    for (int32_t i = 0; i < n_layers; ++i) order_out[i] = n_layers - 1 - i;
    return QV2_OK;
  }
  if (kind != QV2_ORDER_WEIGHT_SQNR) return QV2_ERR_SCHEME;
  if (!w_sqnr_db) return QV2_ERR_NULL;
  for (int32_t i = 0; i < n_layers; ++i) {
    if (std::isnan(w_sqnr_db[i])) return QV2_ERR_NONFINITE;
    order_out[i] = i;
  }
  std::stable_sort(order_out, order_out + n_layers,
                   [&](int32_t a, int32_t b) { return w_sqnr_db[a] < w_sqnr_db[b]; });
  return QV2_OK;
}

// Eq. 17 with bits in {8, 32}; the layers are summed in index order.
static double bops_reduction(const double* macs, const uint8_t* keep, int32_t n) {
  double total = 0.0, mixed = 0.0;
  for (int32_t i = 0; i < n; ++i) {
    total += 32.0 * macs[i];
    mixed += (keep[i] ? 32.0 : 8.0) * macs[i];
  }
  return (1.0 - mixed / total) * 100.0;
}

qv2_status qv2_bops_reduction_pct(const double* macs, const uint8_t* keep_fp32, int32_t n_layers,
                                  double* pct_out) {
  if (!macs || !keep_fp32 || !pct_out) return QV2_ERR_NULL;
  if (n_layers <= 0) return QV2_ERR_SHAPE;
  bool any = false;
  for (int32_t i = 0; i < n_layers; ++i) {
    if (!std::isfinite(macs[i]) || macs[i] < 0.0) return QV2_ERR_NONFINITE;
    any = any || macs[i] > 0.0;
  }
  if (!any) return QV2_ERR_NONFINITE;
  *pct_out = bops_reduction(macs, keep_fp32, n_layers);
  return QV2_OK;
}

qv2_status qv2_bops_select(const int32_t* order, const double* macs, int32_t n_layers,
                           double target_pct, uint8_t* keep_fp32_out, int32_t* n_keep_out,
                           double* achieved_pct_out) {
  return guarded([&]() -> qv2_status {
    if (!order || !macs || !keep_fp32_out) return QV2_ERR_NULL;
    if (n_layers <= 0) return QV2_ERR_SHAPE;
    std::vector<char> seen(n_layers, 0);
    bool any = false;
    for (int32_t i = 0; i < n_layers; ++i) {
      if (order[i] < 0 || order[i] >= n_layers || seen[order[i]]) return QV2_ERR_SHAPE;
      seen[order[i]] = 1;
      if (!std::isfinite(macs[i]) || macs[i] < 0.0) return QV2_ERR_NONFINITE;
      any = any || macs[i] > 0.0;
    }
    if (!any || std::isnan(target_pct)) return QV2_ERR_NONFINITE;
    std::memset(keep_fp32_out, 0, static_cast<size_t>(n_layers));
    int32_t kept = 0;
    for (int32_t k = 0; k < n_layers; ++k) {
      const int32_t l = order[k];
      keep_fp32_out[l] = 1;
      if (bops_reduction(macs, keep_fp32_out, n_layers) < target_pct) { keep_fp32_out[l] = 0; break; }
      ++kept;
    }
    if (n_keep_out) *n_keep_out = kept;
    if (achieved_pct_out) *achieved_pct_out = bops_reduction(macs, keep_fp32_out, n_layers);
    return QV2_OK;
  });
}

// Sec. 4 step 5: bit-width per layer as a text table.
qv2_status qv2_write_config(const char* path, const uint8_t* keep_fp32, const char* const* layer_names,
                            int32_t n_layers) {
  if (!path || !keep_fp32) return QV2_ERR_NULL;
  if (n_layers <= 0) return QV2_ERR_SHAPE;
  if (layer_names)
    for (int32_t i = 0; i < n_layers; ++i) {
      if (!layer_names[i]) return QV2_ERR_NULL;
      if (std::strpbrk(layer_names[i], ",\n\r")) return QV2_ERR_SHAPE;
    }
  std::FILE* f = std::fopen(path, "w");
  if (!f) return QV2_ERR_IO;
  bool ok = std::fputs("layer,name,bits\n", f) >= 0;
  for (int32_t i = 0; ok && i < n_layers; ++i) {
    const int bits = keep_fp32[i] ? 32 : 8;
    if (layer_names) ok = std::fprintf(f, "%d,%s,%d\n", i, layer_names[i], bits) > 0;
    else ok = std::fprintf(f, "%d,layer%d,%d\n", i, i, bits) > 0;
  }
  if (std::fclose(f) != 0) ok = false;
  return ok ? QV2_OK : QV2_ERR_IO;
}

// Sec. 6.5: layers of one fusion group move as a block to the position of the group's most
// sensitive member; list order is kept inside a block and between blocks.
qv2_status qv2_regroup_for_fusion(const int32_t* order, const int32_t* group_id, int32_t n_layers,
                                  int32_t* order_out) {
  return guarded([&]() -> qv2_status {
    if (!order || !group_id || !order_out) return QV2_ERR_NULL;
    if (n_layers <= 0) return QV2_ERR_SHAPE;
    std::vector<char> seen(n_layers, 0), placed(n_layers, 0);
    for (int32_t i = 0; i < n_layers; ++i) {
      if (order[i] < 0 || order[i] >= n_layers || seen[order[i]]) return QV2_ERR_SHAPE;
      seen[order[i]] = 1;
    }
    int32_t w = 0;
    for (int32_t i = 0; i < n_layers; ++i) {
      if (placed[order[i]]) continue;
      const int32_t g = group_id[order[i]];
      for (int32_t k = i; k < n_layers; ++k) {
        const int32_t l = order[k];
        if (!placed[l] && group_id[l] == g) { order_out[w++] = l; placed[l] = 1; }
      }
    }
    return QV2_OK;
  });
}

const char* qv2_status_string(qv2_status s) {
  switch (s) {
    case QV2_OK: return "ok";
    case QV2_ERR_NULL: return "null pointer";
    case QV2_ERR_SHAPE: return "bad shape or count";
    case QV2_ERR_SCHEME: return "unknown quantization scheme";
    case QV2_ERR_WORKSPACE: return "workspace too small";
    case QV2_ERR_NONFINITE: return "non-finite value";
    case QV2_ERR_HIP: return "HIP runtime error";
    case QV2_ERR_ALIGN: return "misaligned pointer";
    case QV2_ERR_IO: return "file could not be written";
    case QV2_ERR_NOMEM: return "out of host memory";
    case QV2_ERR_STATE: return "plan not in the state this call needs";
  }
  return "unknown status";
}

}  // extern "C"
