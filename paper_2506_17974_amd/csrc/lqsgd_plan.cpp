// Host-side planning: validation, HBM layout, work lists.  No HIP calls.
#include "lqsgd_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>

namespace lqsgd {

namespace {

// Work-list sizes below have measured defaults.  Only a build with -DLQSGD_TUNING (for sweeps of
// these sizes) lets an environment variable override them; the normal build reads no environment.
int64_t env_i64(const char* name, int64_t dflt) {
#ifdef LQSGD_TUNING
  const char* s = std::getenv(name);
  if (!s || !*s) return dflt;
  char* end = nullptr;
  long long v = std::strtoll(s, &end, 10);
  return (end && *end == 0 && v > 0) ? (int64_t)v : dflt;
#else
  (void)name;
  return dflt;
#endif
}

int pad_rank(int r) {
  int p = 1;
  while (p < r) p <<= 1;
  return p;
}

}  // namespace

void quantiser_tables(int bits, double alpha, std::vector<float>& thr, std::vector<float>& lev) {
  thr.clear();
  lev.clear();
  if (bits <= 0) return;
  const int lv = (1 << bits) - 1;
  const double l1a = std::log1p(alpha);
  // Eq. (6) at the level q = k/lv, and at the midpoint between two levels.
  for (int k = 0; k <= lv; ++k) lev.push_back((float)(std::expm1((double)k / lv * l1a) / alpha));
  for (int k = 0; k < lv; ++k) thr.push_back((float)(std::expm1((k + 0.5) / lv * l1a) / alpha));
  lev[lv] = 1.0f;   // (1+alpha)^1 - 1 = alpha exactly: the top level is the scale itself
}

int Plan::build(const lqsgd_config* c, const lqsgd_layer* ls, int32_t n_layers) {
  char buf[256];
  if (!c || !ls) { err = "NULL config or layer list"; return LQSGD_EINVAL; }
  if (n_layers < 1) { err = "n_layers must be >= 1"; return LQSGD_EINVAL; }
  if (c->rank < 1 || c->rank > LQSGD_MAX_RANK) {
    std::snprintf(buf, sizeof buf, "rank %d outside 1..%d", c->rank, LQSGD_MAX_RANK);
    err = buf;
    return c->rank < 1 ? LQSGD_EINVAL : LQSGD_EUNSUPPORTED;
  }
  if (c->bits_p < 0 || c->bits_p > 8 || c->bits_q < 0 || c->bits_q > 8) {
    err = "bits_p / bits_q must be 0 (off) or 1..8";
    return LQSGD_EINVAL;
  }
  if (c->workers < 1 || c->workers > LQSGD_MAX_WORKERS) {
    std::snprintf(buf, sizeof buf, "workers %d outside 1..%d", c->workers, LQSGD_MAX_WORKERS);
    err = buf;
    return LQSGD_EINVAL;
  }
  if (!(c->alpha > 0.0f) || !std::isfinite(c->alpha)) { err = "alpha must be finite and > 0"; return LQSGD_EINVAL; }
  if (c->flags & ~(LQSGD_FLAG_EAGER_RESIDUAL | LQSGD_FLAG_AGGREGATE_FIRST | LQSGD_FLAG_BF16_GRADIENTS | LQSGD_FLAG_NO_COOPERATIVE_LAUNCH)) { err = "unknown config flags"; return LQSGD_EINVAL; }
  agg_first = (c->flags & LQSGD_FLAG_AGGREGATE_FIRST) != 0;
  cfg = *c;
  W = c->workers;
  n_all = n_layers;
  layers.clear(); vecs.clear(); kind_of.clear();
  tilesA.clear(); tilesAG.clear(); tilesB.clear(); tilesBM.clear(); tilesG.clear(); tilesXP.clear(); tilesXQ.clear(); tilesRQ.clear(); tilesRP.clear(); tilesV.clear();

  int max_r = 1;
  max_rows = 0;
  matrix_elements = 0;
  for (int i = 0; i < n_layers; ++i) {
    const lqsgd_layer& l = ls[i];
    if (l.rows < 1 || l.cols < 1) {
      std::snprintf(buf, sizeof buf, "layer %d: rows and cols must be >= 1", i);
      err = buf;
      return LQSGD_ESHAPE;
    }
    if ((int64_t)l.rows * l.cols >= ((int64_t)1 << 31)) {
      std::snprintf(buf, sizeof buf, "layer %d: rows*cols must be < 2^31", i);
      err = buf;
      return LQSGD_ESHAPE;
    }
    if (l.flags & ~LQSGD_LAYER_VECTOR) {
      std::snprintf(buf, sizeof buf, "layer %d: unknown flags", i);
      err = buf;
      return LQSGD_EINVAL;
    }
    if (l.flags & LQSGD_LAYER_VECTOR) {
      if (l.cols != 1) {
        std::snprintf(buf, sizeof buf, "layer %d: a VECTOR layer needs cols == 1", i);
        err = buf;
        return LQSGD_ESHAPE;
      }
      VecDesc v{};
      v.len = l.rows;
      v.gidx = i;
      kind_of.push_back(-(int32_t)vecs.size() - 1);
      vecs.push_back(v);
    } else {
      LayerDesc d{};
      d.rows = l.rows;
      d.cols = l.cols;
      d.r = std::min(c->rank, std::min(l.rows, l.cols));
      d.vec = (l.cols % 4 == 0) ? 4 : 1;
      d.gidx = i;
      d.np_el = d.rows * d.r;
      d.nq_el = d.cols * d.r;
      d.np_pad = (int32_t)round_up(d.np_el, 16);
      d.nq_pad = (int32_t)round_up(d.nq_el, 16);
      max_r = std::max(max_r, d.r);
      max_rows = std::max(max_rows, d.rows);
      matrix_elements += (int64_t)d.rows * d.cols;
      kind_of.push_back((int32_t)layers.size());
      layers.push_back(d);
    }
  }
  L = (int32_t)layers.size();
  V = (int32_t)vecs.size();
  RP = pad_rank(max_r);
  max_rank = max_r;
  mfma_a = RP >= env_i64("LQSGD_MFMA_A_MIN_RP", 16);
  mfma = RP >= env_i64("LQSGD_MFMA_MIN_RP", 32);   // measured: at rank pad 16 the vector kernel is still faster

  // ---- tile sizes --------------------------------------------------------
  // A launch wants several times 256 CUs x 16 wavefronts of work items, each
  // long enough to amortise its set-up; huge jobs get larger items so that the
  // work lists stay small.
  const int64_t total = matrix_elements * W;
  const int64_t tgtA = env_i64("LQSGD_TILE_A", std::min<int64_t>(131072, std::max<int64_t>(2048, total / 49152)));
  const int64_t tgtB = env_i64("LQSGD_TILE_B", std::min<int64_t>(524288, std::max<int64_t>(16384, total / 2730)));   // (floor: small CNN set, sweep 1 17.1 -> 14.7 us against 8192)
  // the G-hat-only pass covers one worker's worth of elements: smaller items keep its grid wide
  const int64_t tgtG = env_i64("LQSGD_TILE_G", std::min<int64_t>(tgtB, std::max<int64_t>(4096, matrix_elements / 2730)));
  // column segments: at most 1024 columns (2048 at rank pad 32, where fewer, longer segments save
  // more in partial planes and Gram-Schmidt input than they cost in sweep 0)
  const int64_t segmax4 = env_i64("LQSGD_SEGMAX", RP >= 32 ? 2048 : 1024);

  int64_t m_acc = 0, p_acc = 0, q_acc = 0, pp_acc = 0, qp_acc = 0;
  int64_t mp_acc = 0, sp_acc = 0, mq_acc = 0, sq_acc = 0;
  int64_t ppd_acc = 0, qpd_acc = 0;
  padded = false;
  wire_bytes = 0;
  // the reduce passes: items of 1024 .. 8192 elements, as large as still leaves about 512 of them
  // (one atomic maximum per item on a cell per (layer, worker); several loads in flight per thread)
  auto reduce_chunk = [&](bool q) {
    int64_t total = 0;
    for (const LayerDesc& d : layers) total += q ? d.nq_el : d.np_el;
    return (int32_t)(1024 * std::min<int64_t>(8, std::max<int64_t>(1, total * W / (1024 * 512))));
  };
  const int32_t rq_chunk = reduce_chunk(true), rp_chunk = reduce_chunk(false);
  for (int li = 0; li < L; ++li) {
    LayerDesc& d = layers[li];
    const int cw = kWave * d.vec;
    const int64_t segmax = std::max<int64_t>(cw, d.vec == 4 ? round_up(segmax4, cw) : 256);
    int nseg = (int)((d.cols + segmax - 1) / segmax);
    d.segw = (int32_t)round_up((d.cols + nseg - 1) / nseg, cw);
    d.nseg = (d.cols + d.segw - 1) / d.segw;
    const int rowgrp = mfma_a ? 32 : kRowsPerGroup;      // a matrix-core item is one 32-row tile
    const int64_t seg_elems = (int64_t)rowgrp * std::min(d.segw, d.cols);
    int64_t ng = mfma_a ? 1 : std::max<int64_t>(1, (tgtA + seg_elems / 2) / seg_elems);
    const int32_t trows = (int32_t)std::min<int64_t>(round_up(d.rows, rowgrp), ng * rowgrp);

    // sweeps 1 / 2 on the vector units: row blocks of rbb_v rows
    int64_t rbb = std::max<int64_t>(4, round_up(std::max<int64_t>(1, tgtB / cw), 4));
    int32_t rbb_v = (int32_t)std::min<int64_t>(rbb, round_up(d.rows, 4));
    int32_t nrb_v = (d.rows + rbb_v - 1) / rbb_v;
    // equal blocks: 8192 rows in blocks of 1536 would end in a block of 512
    rbb_v = (int32_t)std::min<int64_t>(rbb_v, round_up((d.rows + nrb_v - 1) / nrb_v, 4));
    nrb_v = (d.rows + rbb_v - 1) / rbb_v;
    // Layers of moderate height take one row block per column chunk: sweep 1 then writes Q_w itself
    // (no partial planes, no reduce pass for this layer), and measured on the ResNet-18-shaped set
    // it streams as fast with 512-row items as with 128-row ones (63 us either way).
    // Not where that would leave the launch with too few items: at most four times the size the
    // work list aims for (a 1024-row layer of a small set keeps its row blocks).
    if (!mfma && (int64_t)d.rows * cw <= env_i64("LQSGD_DIRECT_Q_MAX", 262144) && d.rows <= 4 * rbb) {
      rbb_v = (int32_t)round_up(d.rows, 4);
      nrb_v = 1;
    }
    // the partial planes of Q belong to whichever kernel runs sweep 1
    if (mfma) {
      const int64_t rbm = env_i64("LQSGD_TILE_BM", std::min<int64_t>(2048, std::max<int64_t>(256, total / (49152 * 16))));
      d.rbb = (int32_t)std::min<int64_t>(round_up(rbm, 2), round_up(d.rows, 2));
    } else {
      d.rbb = rbb_v;
    }
    d.nrb = (d.rows + d.rbb - 1) / d.rbb;
    d.direct_q = (!mfma && d.nrb == 1) ? 1 : 0;
    const int nchunk = (d.cols + cw - 1) / cw;

    d.m_off = m_acc;   m_acc += round_up((int64_t)d.rows * d.cols, 64);
    d.p_off = p_acc;   p_acc += round_up(d.np_el, 64);
    d.q_off = q_acc;   q_acc += round_up(d.nq_el, 64);
    d.ppart_off = pp_acc; pp_acc += (int64_t)d.nseg * d.np_pad;
    d.qpart_off = qp_acc; qp_acc += d.direct_q ? 0 : (int64_t)d.nrb * d.nq_pad;   // no partial planes where sweep 1 stores Q_w itself
    d.ppad_off = ppd_acc; ppd_acc += round_up((int64_t)d.rows * RP, 64);
    d.qpad_off = qpd_acc; qpd_acc += round_up((int64_t)d.cols * RP, 64);
    if (mfma_a && d.vec == 4 && d.r < RP && env_i64("LQSGD_NO_PAD_OPERANDS", 0) == 0) padded = true;
    const int64_t gp = (d.np_el + kXGroup - 1) / kXGroup, gq = (d.nq_el + kXGroup - 1) / kXGroup;
    d.magp_off = mp_acc; mp_acc += round_up(gp * std::max(1, cfg.bits_p), 16);
    d.sgnp_off = sp_acc; sp_acc += round_up(gp, 16);
    d.magq_off = mq_acc; mq_acc += round_up(gq * std::max(1, cfg.bits_q), 16);
    d.sgnq_off = sq_acc; sq_acc += round_up(gq, 16);

    wire_bytes += cfg.bits_p ? ((int64_t)d.np_el * cfg.bits_p + 7) / 8 + gp + 4 : 4 * (int64_t)d.np_el;
    wire_bytes += cfg.bits_q ? ((int64_t)d.nq_el * cfg.bits_q + 7) / 8 + gq + 4 : 4 * (int64_t)d.nq_el;

    for (int w = 0; w < W; ++w) {
      const int32_t lw = li * W + w;
      for (int32_t row0 = 0; row0 < d.rows; row0 += trows)
        for (int32_t s = 0; s < d.nseg; ++s) {
          tilesA.push_back(Tile{lw, row0, std::min(trows, d.rows - row0), s});
          if (w == 0) tilesAG.push_back(tilesA.back());
        }
      for (int32_t rb = 0; rb < nrb_v; ++rb)
        for (int32_t ch = 0; ch < nchunk; ++ch)
          tilesB.push_back(Tile{lw, rb * rbb_v, std::min(rbb_v, d.rows - rb * rbb_v), ch});
      if (w == 0) {
        const int32_t rbg = (int32_t)std::min<int64_t>(round_up(std::max<int64_t>(1, tgtG / cw), 4), round_up(d.rows, 4));
        for (int32_t row0 = 0; row0 < d.rows; row0 += rbg)
          for (int32_t ch = 0; ch < nchunk; ++ch)
            tilesG.push_back(Tile{lw, row0, std::min(rbg, d.rows - row0), ch});
      }
      if (mfma)
        for (int32_t rb = 0; rb < d.nrb; ++rb)
          for (int32_t cg = 0; cg < (d.cols + kMfmaCols - 1) / kMfmaCols; ++cg)
            tilesBM.push_back(Tile{lw, rb * d.rbb, std::min(d.rbb, d.rows - rb * d.rbb), cg});
      if (!d.direct_q)
        for (int32_t e = 0; e < d.nq_el; e += rq_chunk) tilesRQ.push_back(RTile{lw, e, std::min(rq_chunk, d.nq_el - e)});
      if (agg_first)
        for (int32_t e = 0; e < d.np_el; e += rp_chunk) tilesRP.push_back(RTile{lw, e, std::min(rp_chunk, d.np_el - e)});
    }
    for (int32_t g = 0; g < gp; g += kXBlockGroups) tilesXP.push_back(XTile{li, g});
    for (int32_t g = 0; g < gq; g += kXBlockGroups) tilesXQ.push_back(XTile{li, g});
  }
  m_stride = round_up(m_acc, 64);
  p_stride = round_up(p_acc, 64);
  q_stride = round_up(q_acc, 64);
  ppart_stride = round_up(pp_acc, 64);
  qpart_stride = round_up(qp_acc, 64);
  magp_stride = round_up(mp_acc, 64);
  sgnp_stride = round_up(sp_acc, 64);
  magq_stride = round_up(mq_acc, 64);
  sgnq_stride = round_up(sq_acc, 64);
  ppad_total = padded ? ppd_acc : 0;
  qpad_total = padded ? qpd_acc : 0;

  int64_t v_acc = 0;
  for (int vi = 0; vi < V; ++vi) {
    vecs[vi].off = v_acc;
    for (int32_t e = 0; e < vecs[vi].len; e += 1024) tilesV.push_back(VTile{vi, e});
    v_acc += round_up(vecs[vi].len, 64);
  }
  v_total = v_acc;

  const int64_t tile_bytes = (int64_t)(tilesA.size() + tilesAG.size() + tilesB.size() + tilesBM.size() + tilesG.size()) * sizeof(Tile) +
                             (int64_t)(tilesXP.size() + tilesXQ.size()) * sizeof(XTile) +
                             (int64_t)(tilesRQ.size() + tilesRP.size()) * sizeof(RTile) + (int64_t)tilesV.size() * sizeof(VTile);
  device_bytes = 4 * ((int64_t)W * (m_stride + 2 * p_stride + q_stride + ppart_stride + qpart_stride) +
                      p_stride + q_stride + ppad_total + qpad_total + v_total + 2 * (int64_t)W * std::max(L, 1) +
                      6 * (int64_t)W * std::max(L, 1) * ((max_rows + 255) / 256) * RP) +
                 (int64_t)W * (magp_stride + sgnp_stride + magq_stride + sgnq_stride) + tile_bytes +
                 (int64_t)L * sizeof(LayerDesc) + (int64_t)V * sizeof(VecDesc) +
                 (int64_t)(W + 1) * n_all * 8 + 4 * 4 * 256;
  if (tilesA.size() > 0x7fffffff / 4 || tilesB.size() > 0x7fffffffu) {
    err = "work list too long";
    return LQSGD_EUNSUPPORTED;
  }
  return LQSGD_OK;
}

}  // namespace lqsgd
