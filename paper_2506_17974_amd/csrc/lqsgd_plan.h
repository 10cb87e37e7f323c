// Host-side planning for the LQ-SGD compressor: layer table, buffer layout in
// HBM and the flattened work lists of every kernel.  Pure C++ (no HIP calls),
// so it can be exercised on a machine without a GPU.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "lqsgd.h"

namespace lqsgd {

constexpr int kWave = 64;
constexpr int kRowsPerGroup = 8;   // rows a wavefront carries through one column pass of sweep 0
constexpr int kMfmaCols = 512;     // columns one workgroup of the matrix-core sweep 1 covers (4 waves x 4 strips x 32)
constexpr int kXGroup = 8;         // elements one lane quantises / packs (b bytes + 1 sign byte)
constexpr int kXBlockGroups = 32;  // groups of 8 elements one exchange workgroup covers
constexpr int kFactorSlack = 64;   // readable floats after the last row of every factor buffer (loaders of ranks below their pad overrun)

// One matrix layer as the kernels see it.  Offsets are in elements (floats)
// from the start of a per-worker slab unless they say bytes.
struct LayerDesc {
  int32_t rows, cols, r, vec;   // vec = 4 when rows are 16-byte aligned (cols % 4 == 0), else 1
  int32_t segw, nseg;           // sweep 0: column segment width (multiple of 64*vec) and count
  int32_t rbb, nrb;             // sweeps 1, 2: rows per row block and count
  int32_t gidx;                 // position in the caller's tensor list
  int32_t np_el, nq_el;         // rows*r, cols*r
  int32_t np_pad, nq_pad;       // the same rounded up to 16 elements (stride of the partial planes)
  int32_t direct_q;             // sweep 1 covers all rows in one block and writes Q_w (and its absmax) itself: no partial planes, no reduce
  int64_t m_off;                // into E / M          (worker stride m_stride)
  int64_t p_off;                // into rows x r slabs (worker stride p_stride)
  int64_t q_off;                // into cols x r slabs (worker stride q_stride)
  int64_t ppart_off;            // nseg planes of np_pad (worker stride ppart_stride)
  int64_t qpart_off;            // nrb planes of nq_pad  (worker stride qpart_stride)
  int64_t magp_off, sgnp_off;   // bytes (worker strides magp_stride, sgnp_stride)
  int64_t magq_off, sgnq_off;   // bytes
  int64_t ppad_off, qpad_off;   // into the copies of P-bar / Q-bar with rows padded to RP ranks (Plan::padded)
};

struct VecDesc {
  int32_t len, gidx;
  int64_t off;                  // into the vmean buffer
};

// Work item of a streaming sweep.  lw = layer * W + worker.
// sweep 0: one wavefront; rows [row0, row0+nrows), column segment `aux`.
// sweeps 1, 2: one workgroup; rows [row0, row0+nrows), column chunk `aux` (64*vec wide).
struct Tile {
  int32_t lw, row0, nrows, aux;
};
struct XTile {   // exchange kernels: kXBlockGroups groups of 8 elements starting at group grp0 of `layer`
  int32_t layer, grp0;
};
struct RTile {   // reduce_q: n elements of (layer, worker) starting at el0 (n <= 8192, el0 a multiple of 1024)
  int32_t lw, el0, n;
};
struct VTile {   // vector_mean: 1024 elements of vector `vec` starting at el0
  int32_t vec, el0;
};

struct Plan {
  lqsgd_config cfg{};
  int32_t n_all = 0;            // tensors in the caller's list
  int32_t W = 0, L = 0, V = 0;  // workers, matrix layers, vector layers
  int32_t RP = 0;               // register rank: smallest of 1,2,4,8,16,32 >= max layer rank
  int32_t max_rows = 0;         // largest row count of a matrix layer
  int32_t max_rank = 0;         // largest effective rank of a matrix layer
  bool mfma = false;            // sweep 1 runs on the matrix cores (rank pad 32)
  bool mfma_a = false;          // sweeps 0 and 2 run on the matrix cores (rank pad >= 16): 32-row work items
  std::vector<LayerDesc> layers;
  std::vector<VecDesc> vecs;
  std::vector<int32_t> kind_of;    // per caller index: >= 0 matrix index, < 0 -(vector index) - 1
  std::vector<Tile> tilesA, tilesB;
  std::vector<Tile> tilesAG;       // worker 0's items of tilesA (G-hat pass of the matrix-core path)
  std::vector<Tile> tilesBM;       // sweep 1 on the matrix cores (rank pad >= 16): row block x 128-column group
  std::vector<Tile> tilesG;        // worker 0's items of tilesB: one pass over every layer (G-hat only)
  std::vector<XTile> tilesXP, tilesXQ;
  std::vector<RTile> tilesRQ;
  std::vector<RTile> tilesRP;      // aggregate-first order: reduce of the P partials (1024 elements each)
  bool agg_first = false;          // LQSGD_FLAG_AGGREGATE_FIRST
  // Some layer that the matrix-core sweeps 0 / 2 handle has fewer ranks than the register pad: these
  // sweeps then read P-bar and Q-bar from copies whose rows are padded with zeros to RP ranks
  // (16-byte aligned rows, no rank tests in the loops); ppad_total / qpad_total floats.
  bool padded = false;
  int64_t ppad_total = 0, qpad_total = 0;
  std::vector<VTile> tilesV;
  int64_t m_stride = 0, p_stride = 0, q_stride = 0, ppart_stride = 0, qpart_stride = 0;
  int64_t magp_stride = 0, sgnp_stride = 0, magq_stride = 0, sgnq_stride = 0, v_total = 0;
  int64_t device_bytes = 0, wire_bytes = 0, matrix_elements = 0;
  std::string err;

  // Returns LQSGD_OK or a negative status with `err` set.
  int build(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers);
};

// Quantiser tables of Section 4.1 for one bit width, computed in double and
// rounded to fp32: thr[k] = decision threshold between levels k and k+1 in the
// normalised magnitude u = |x|/s, k < 2^b - 1; lev[k] = dequantised magnitude
// of level k, k < 2^b.
void quantiser_tables(int bits, double alpha, std::vector<float>& thr, std::vector<float>& lev);

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace lqsgd
