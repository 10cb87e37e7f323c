// gfx950 kernels of the LQ-SGD compressor (Algorithm 1 of the paper, loop body).
//
// Three streaming sweeps over the W x (rows x cols) gradient data, each one
// batched launch over all layers and workers, and small kernels on the
// rows x r / cols x r factors between them:
//
//   add_project   M = G + E (stored over E), P partials = M Q        12 B / element
//   orth          sum partials, Gram-Schmidt, absmax                 factors only
//   exchange(P)   log-quantise, pack, dequantise, mean over workers  factors only
//   back_project  Q partials = M^T P-bar                              4 B / element
//   reduce_q      sum partials, absmax                               factors only
//   exchange(Q)   as exchange(P)                                     factors only
//   residual      E = M - P-bar Q-bar^T (and G-hat once per layer)    8 B / element
//
// Lanes own columns in every sweep (one float4 per lane per row: a wavefront
// reads 1 KiB of a row per instruction); the r-wide factor slice of a lane's
// columns lives in registers; rows of the other factor are wave-uniform.
// All reductions have a fixed order, so results are bit-identical run to run.
#include "lqsgd_kernels.h"

#include <cfloat>

namespace lqsgd {
namespace {

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
template <int V>
struct Pk {
  float v[V];
};

template <int V>
__device__ __forceinline__ Pk<V> ldv(const float* p);
template <>
__device__ __forceinline__ Pk<4> ldv<4>(const float* p) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  return Pk<4>{{t.x, t.y, t.z, t.w}};
}
template <>
__device__ __forceinline__ Pk<1> ldv<1>(const float* p) {
  return Pk<1>{{*p}};
}
template <int V>
__device__ __forceinline__ void stv(float* p, const Pk<V>& x);
template <>
__device__ __forceinline__ void stv<4>(float* p, const Pk<4>& x) {
  *reinterpret_cast<float4*>(p) = make_float4(x.v[0], x.v[1], x.v[2], x.v[3]);
}
template <>
__device__ __forceinline__ void stv<1>(float* p, const Pk<1>& x) {
  *p = x.v[0];
}

// Factor slice of VEC consecutive columns starting at column c of a cols x r
// row-major factor F, as s[v*RP + k].  `exact` (r == RP) is the fast path.
template <int RP, int VEC>
__device__ __forceinline__ void load_slice(const float* __restrict__ F, int c, int r, bool exact,
                                           float (&s)[VEC * RP]) {
  if (exact) {
    const float* base = F + (size_t)c * RP;
    if constexpr ((VEC * RP) % 4 == 0) {
#pragma unroll
      for (int i = 0; i < VEC * RP / 4; ++i) {
        const float4 t = reinterpret_cast<const float4*>(base)[i];
        s[4 * i + 0] = t.x; s[4 * i + 1] = t.y; s[4 * i + 2] = t.z; s[4 * i + 3] = t.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < VEC * RP; ++i) s[i] = base[i];
    }
  } else {
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int k = 0; k < RP; ++k) s[v * RP + k] = (k < r) ? F[(size_t)(c + v) * r + k] : 0.0f;
  }
}

template <int RP, int VEC>
__device__ __forceinline__ void store_slice(float* __restrict__ F, int c, int r, bool exact,
                                            const float (&s)[VEC * RP]) {
  if (exact) {
    float* base = F + (size_t)c * RP;
    if constexpr ((VEC * RP) % 4 == 0) {
#pragma unroll
      for (int i = 0; i < VEC * RP / 4; ++i)
        reinterpret_cast<float4*>(base)[i] = make_float4(s[4 * i], s[4 * i + 1], s[4 * i + 2], s[4 * i + 3]);
    } else {
#pragma unroll
      for (int i = 0; i < VEC * RP; ++i) base[i] = s[i];
    }
  } else {
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) F[(size_t)(c + v) * r + k] = s[v * RP + k];
  }
}

// Wave-uniform row of a rows x r factor into p[k] (zero beyond r).
template <int RP>
__device__ __forceinline__ void load_row(const float* __restrict__ F, int row, int r, bool exact, float (&p)[RP]) {
  if (exact) {
    const float* b = F + (size_t)row * RP;
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = b[k];
  } else {
    const float* b = F + (size_t)row * r;
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = (k < r) ? b[k] : 0.0f;
  }
}

// Sum of N per-lane values over the 64 lanes of a wavefront, N a power of two.
// Each butterfly step exchanges half of the still-live values, so the cost is
// about N shuffles instead of 6 N.  On return lane l holds, in v[0 .. max(1,N/64)),
// the totals of the values with index l*(N/64)+i (N >= 64), or of index
// l >> (6 - log2 N) replicated over 64/N neighbouring lanes (N < 64).
template <int NT, int LIVE, int OFF>
__device__ __forceinline__ void transpose_reduce(float (&v)[NT], int lane) {
  if constexpr (OFF >= 1) {
    if constexpr (LIVE > 1) {
      constexpr int H = LIVE / 2;
      const bool hi = (lane & OFF) != 0;
#pragma unroll
      for (int i = 0; i < H; ++i) {
        const float keep = hi ? v[i + H] : v[i];
        const float send = hi ? v[i] : v[i + H];
        v[i] = keep + __shfl_xor(send, OFF, kWave);
      }
      transpose_reduce<NT, H, OFF / 2>(v, lane);
    } else {
      v[0] += __shfl_xor(v[0], OFF, kWave);
      transpose_reduce<NT, 1, OFF / 2>(v, lane);
    }
  }
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}

constexpr int log2c(int n) { return n <= 1 ? 0 : 1 + log2c(n / 2); }

// ---------------------------------------------------------------------------
// sweep 0: M = G + E (Eq. (9)),  P_w partial = M_w Q  (Algorithm 1, "P <- G'Q")
// One wavefront per work item: rows [row0, row0+nrows) x columns [col0, col1).
// ---------------------------------------------------------------------------
template <int RP, int VEC, int RT>
__device__ __forceinline__ void add_project_tile(const float* __restrict__ G, float* __restrict__ M,
                                                 const float* __restrict__ Q, float* __restrict__ Pp,
                                                 int cols, int r, int row0, int nrows, int col0, int col1,
                                                 int lane) {
  constexpr int N = RT * RP;
  const bool exact = (r == RP);
  for (int rg = 0; rg < nrows; rg += RT) {
    const int nr = min(RT, nrows - rg);
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.0f;
    const size_t rowbase = (size_t)(row0 + rg) * cols;
    for (int c = col0 + lane * VEC; c < col1; c += kWave * VEC) {
      float q[VEC * RP];
      load_slice<RP, VEC>(Q, c, r, exact, q);
      Pk<VEC> g[RT], e[RT];
      if (nr == RT) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          g[t] = ldv<VEC>(G + rowbase + (size_t)t * cols + c);
          e[t] = ldv<VEC>(M + rowbase + (size_t)t * cols + c);
        }
      } else {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          if (t < nr) {
            g[t] = ldv<VEC>(G + rowbase + (size_t)t * cols + c);
            e[t] = ldv<VEC>(M + rowbase + (size_t)t * cols + c);
          } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) { g[t].v[v] = 0.0f; e[t].v[v] = 0.0f; }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        Pk<VEC> m;
#pragma unroll
        for (int v = 0; v < VEC; ++v) m.v[v] = g[t].v[v] + e[t].v[v];
        if (t < nr) stv<VEC>(M + rowbase + (size_t)t * cols + c, m);
#pragma unroll
        for (int v = 0; v < VEC; ++v)
#pragma unroll
          for (int k = 0; k < RP; ++k) acc[t * RP + k] = fmaf(m.v[v], q[v * RP + k], acc[t * RP + k]);
      }
    }
    transpose_reduce<N, N, 32>(acc, lane);
    constexpr int NPL = (N >= kWave) ? N / kWave : 1;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      int idx;
      bool writer;
      if constexpr (N >= kWave) {
        idx = lane * NPL + i;
        writer = true;
      } else {
        idx = lane >> (6 - log2c(N));
        writer = (lane & (kWave / N - 1)) == 0;
      }
      const int t = idx / RP, k = idx - t * RP;
      if (writer && t < nr && k < r) Pp[(size_t)(row0 + rg + t) * r + k] = acc[i];
    }
  }
}

template <int RP>
__global__ __launch_bounds__(256) void add_project_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles) {
  constexpr int RT = (RP <= 8) ? 8 : 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  const int t = blockIdx.x * 4 + wave;
  if (t >= ntiles) return;
  const Tile tl = tiles[t];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const float* G = a.grads[(size_t)worker * a.n_all + ld.gidx];
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Q = a.Qbar + ld.q_off;
  float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off + (size_t)tl.aux * ld.np_pad;
  const int col0 = tl.aux * ld.segw;
  const int col1 = min(ld.cols, col0 + ld.segw);
  if (ld.vec == 4)
    add_project_tile<RP, 4, RT>(G, M, Q, Pp, ld.cols, ld.r, tl.row0, tl.nrows, col0, col1, lane);
  else
    add_project_tile<RP, 1, RT>(G, M, Q, Pp, ld.cols, ld.r, tl.row0, tl.nrows, col0, col1, lane);
}

// ---------------------------------------------------------------------------
// orth: P_w = sum of the column-segment partials; modified Gram-Schmidt
// (Algorithm 1, "Orthonormalize"), right-looking: column j is normalised, then
// removed from every later column, which applies the projections to a column
// in the same order as the left-looking form.  One workgroup per (layer,
// worker); a lane owns rows tid, tid+256, ... through all passes, so the only
// communication is the block-wide sums.  Ends with absmax(P_w) -> scaleP.
// ---------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void orth_kernel(DevArgs a) {
  __shared__ float red[2][4][RP];
  __shared__ float redmax[4];
  const int lw = blockIdx.x;
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r, nseg = ld.nseg;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off;
  float* pre = a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  float* orth = a.Porth + (size_t)worker * a.p_stride + ld.p_off;

  for (int row = tid; row < rows; row += 256) {
    float v[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) v[k] = 0.0f;
    for (int s = 0; s < nseg; ++s) {
      const float* src = Pp + (size_t)s * ld.np_pad + (size_t)row * r;
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) v[k] += src[k];
    }
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) {
        pre[(size_t)row * r + k] = v[k];
        orth[(size_t)row * r + k] = v[k];
      }
  }

  for (int j = 0; j < r; ++j) {
    // s[k] = <column j, column k> for every k (entries k < j are not used)
    float s[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) s[k] = 0.0f;
    for (int row = tid; row < rows; row += 256) {
      const float* src = orth + (size_t)row * r;
      const float vj = src[j];
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) s[k] = fmaf(vj, src[k], s[k]);
    }
#pragma unroll
    for (int k = 0; k < RP; ++k) s[k] = wave_sum(s[k]);
    const int b = j & 1;
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < RP; ++k) red[b][wave][k] = s[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RP; ++k) s[k] = (red[b][0][k] + red[b][1][k]) + (red[b][2][k] + red[b][3][k]);
    const float nrm2 = (red[b][0][j] + red[b][1][j]) + (red[b][2][j] + red[b][3][j]);
    const float inv = (nrm2 > FLT_MIN) ? 1.0f / sqrtf(nrm2) : 0.0f;
    for (int row = tid; row < rows; row += 256) {
      float* dst = orth + (size_t)row * r;
      const float qv = dst[j] * inv;
      dst[j] = qv;
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k > j && k < r) dst[k] = fmaf(-(s[k] * inv), qv, dst[k]);
    }
  }

  float mx = 0.0f;
  for (int row = tid; row < rows; row += 256) {
    const float* src = orth + (size_t)row * r;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) mx = fmaxf(mx, fabsf(src[k]));
  }
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0) a.scaleP[(size_t)worker * a.L + layer] = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
}

// ---------------------------------------------------------------------------
// exchange: LogQuantize (Eq. (5) discretised to 2^b levels, Section 4.1),
// pack, LogDequantize (Eq. (6)) and the mean over workers that stands in for
// the All-Reduce.  A lane handles 8 consecutive factor elements of every
// worker: b magnitude bytes + 1 sign byte per worker.
//   kQuantOnly: factors -> packets      kMeanOnly: packets -> mean
//   kFused:     factors -> packets and mean in one pass
// The code of u = |x|/s is the number of thresholds <= u (binary search in
// LDS), which is nearest-level rounding in the q-domain of Eq. (5).
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void exchange_kernel(DevArgs a, const XTile* __restrict__ tiles, int phase) {
  __shared__ float s_thr[256];
  __shared__ float s_lev[256];
  const int bits = phase ? a.bits_q : a.bits_p;
  const int lv = (1 << bits) - 1;
  const int tid = threadIdx.x;
  if (bits > 0) {
    const float* thr = phase ? a.thrQ : a.thrP;
    const float* lev = phase ? a.levQ : a.levP;
    if (tid < lv) s_thr[tid] = thr[tid];
    if (tid <= lv) s_lev[tid] = lev[tid];
  }
  __syncthreads();
  const XTile tl = tiles[blockIdx.x];
  const LayerDesc& ld = a.layers[tl.layer];
  const int n_el = phase ? ld.nq_el : ld.np_el;
  const int g = tl.grp0 + tid;
  const int e0 = g * kXGroup;
  if (e0 >= n_el) return;
  const int nvalid = min(kXGroup, n_el - e0);
  const size_t fstride = phase ? a.q_stride : a.p_stride;
  const float* fac = (phase ? a.Qw + ld.q_off : a.Porth + ld.p_off) + e0;
  uint8_t* mag = (phase ? a.magQ + ld.magq_off : a.magP + ld.magp_off) + (size_t)g * bits;
  uint8_t* sgn = (phase ? a.sgnQ + ld.sgnq_off : a.sgnP + ld.sgnp_off) + g;
  const size_t mstride = phase ? a.magq_stride : a.magp_stride;
  const size_t sstride = phase ? a.sgnq_stride : a.sgnp_stride;
  const float* scale = phase ? a.scaleQ : a.scaleP;

  float acc[kXGroup];
#pragma unroll
  for (int i = 0; i < kXGroup; ++i) acc[i] = 0.0f;

  for (int w = 0; w < a.W; ++w) {
    float x[kXGroup];
    if (MODE != kMeanOnly || bits == 0) {
      const float4 lo = reinterpret_cast<const float4*>(fac + (size_t)w * fstride)[0];
      const float4 hi = reinterpret_cast<const float4*>(fac + (size_t)w * fstride)[1];
      x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
      x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
#pragma unroll
      for (int i = 0; i < kXGroup; ++i)
        if (i >= nvalid) x[i] = 0.0f;
    }
    if (bits == 0) {
      if (MODE != kQuantOnly) {
#pragma unroll
        for (int i = 0; i < kXGroup; ++i) acc[i] += x[i];
      }
      continue;
    }
    const float s = scale[(size_t)w * a.L + tl.layer];
    unsigned long long magbits = 0;
    unsigned sgnbits = 0;
    if (MODE != kMeanOnly) {
#pragma unroll
      for (int i = 0; i < kXGroup; ++i) {
        int k = 0;
        if (s > 0.0f) {
          const float u = fabsf(x[i]) / s;
          int lo = 0, hi = lv;
          while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_thr[mid] <= u) lo = mid + 1; else hi = mid;
          }
          k = lo;
        }
        magbits |= (unsigned long long)k << (i * bits);
        if (x[i] < 0.0f && k > 0) sgnbits |= 1u << i;
      }
      uint8_t* mp = mag + (size_t)w * mstride;
      if (bits == 8) {
        *reinterpret_cast<unsigned long long*>(mp) = magbits;
      } else if (bits == 4) {
        *reinterpret_cast<unsigned*>(mp) = (unsigned)magbits;
      } else if (bits == 2) {
        *reinterpret_cast<unsigned short*>(mp) = (unsigned short)magbits;
      } else {
        for (int bb = 0; bb < bits; ++bb) mp[bb] = (uint8_t)(magbits >> (8 * bb));
      }
      sgn[(size_t)w * sstride] = (uint8_t)sgnbits;
    } else {
      const uint8_t* mp = mag + (size_t)w * mstride;
      for (int bb = 0; bb < bits; ++bb) magbits |= (unsigned long long)mp[bb] << (8 * bb);
      sgnbits = sgn[(size_t)w * sstride];
    }
    if (MODE != kQuantOnly) {
#pragma unroll
      for (int i = 0; i < kXGroup; ++i) {
        const int k = (int)((magbits >> (i * bits)) & (unsigned long long)lv);
        const float val = s * s_lev[k];
        acc[i] += ((sgnbits >> i) & 1u) ? -val : val;
      }
    }
  }
  if (MODE != kQuantOnly) {
    float* out = (phase ? a.Qbar + ld.q_off : a.Pbar + ld.p_off) + e0;
    const float wf = (float)a.W;
#pragma unroll
    for (int i = 0; i < kXGroup; ++i)
      if (i < nvalid) out[i] = acc[i] / wf;
  }
}

// ---------------------------------------------------------------------------
// sweep 1: Q_w partial = M_w^T P-bar over a row block (Algorithm 1,
// "Q <- G'^T P").  One workgroup per (row block, 64*VEC-column chunk); its four
// wavefronts split the rows and combine through LDS in a fixed tree.
// ---------------------------------------------------------------------------
template <int RP, int VEC>
__device__ __forceinline__ void back_project_rows(const float* __restrict__ M, const float* __restrict__ Pb,
                                                  int cols, int r, bool exact, int ra, int rb, int c,
                                                  float (&acc)[VEC * RP]) {
  constexpr int U = 8;
  int i = ra;
  for (; i + U <= rb; i += U) {
    Pk<VEC> m[U];
#pragma unroll
    for (int u = 0; u < U; ++u) m[u] = ldv<VEC>(M + (size_t)(i + u) * cols + c);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float p[RP];
      load_row<RP>(Pb, i + u, r, exact, p);
#pragma unroll
      for (int v = 0; v < VEC; ++v)
#pragma unroll
        for (int k = 0; k < RP; ++k) acc[v * RP + k] = fmaf(m[u].v[v], p[k], acc[v * RP + k]);
    }
  }
  for (; i < rb; ++i) {
    const Pk<VEC> m = ldv<VEC>(M + (size_t)i * cols + c);
    float p[RP];
    load_row<RP>(Pb, i, r, exact, p);
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int k = 0; k < RP; ++k) acc[v * RP + k] = fmaf(m.v[v], p[k], acc[v * RP + k]);
  }
}

template <int RP, int VEC>
__device__ __forceinline__ void back_project_tile(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                                  float* comb, int wave, int lane) {
  constexpr int NV = VEC * RP;
  const int cols = ld.cols, r = ld.r;
  const bool exact = (r == RP);
  const float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  const int c = tl.aux * (kWave * VEC) + lane * VEC;
  const bool active = c < cols;
  const int per = (tl.nrows + 3) >> 2;
  const int ra = min(tl.row0 + wave * per, tl.row0 + tl.nrows);
  const int rb = min(ra + per, tl.row0 + tl.nrows);
  float acc[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) acc[i] = 0.0f;
  if (active) back_project_rows<RP, VEC>(M, Pb, cols, r, exact, ra, rb, c, acc);
  // (wave 0 + wave 2) + (wave 1 + wave 3)
  if (wave >= 2) {
#pragma unroll
    for (int i = 0; i < NV; ++i) comb[(wave - 2) * (kWave * NV) + i * kWave + lane] = acc[i];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] += comb[wave * (kWave * NV) + i * kWave + lane];
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int i = 0; i < NV; ++i) comb[i * kWave + lane] = acc[i];
  }
  __syncthreads();
  if (wave == 0 && active) {
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] += comb[i * kWave + lane];
    float* Qp = a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off + (size_t)(tl.row0 / ld.rbb) * ld.nq_pad;
    store_slice<RP, VEC>(Qp, c, r, exact, acc);
  }
}

template <int RP>
__global__ __launch_bounds__(256) void back_project_kernel(DevArgs a, const Tile* __restrict__ tiles) {
  __shared__ float comb[2 * kWave * 4 * RP];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (blockIdx.x == 0) {   // absmax accumulators of reduce_q start from zero
    for (int i = threadIdx.x; i < a.W * a.L; i += 256) a.scaleQ[i] = 0.0f;
  }
  const Tile tl = tiles[blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  if (ld.vec == 4)
    back_project_tile<RP, 4>(a, ld, tl, worker, comb, wave, lane);
  else
    back_project_tile<RP, 1>(a, ld, tl, worker, comb, wave, lane);
}

// ---------------------------------------------------------------------------
// reduce_q: Q_w = sum over row blocks of the partials (fixed order), and
// absmax(Q_w) -> scaleQ.  The max over workgroups goes through an integer
// atomic max on the float's bit pattern (non-negative floats order like
// unsigned integers), which is exact and order-independent.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void reduce_q_kernel(DevArgs a, const RTile* __restrict__ tiles) {
  __shared__ float redmax[4];
  const RTile tl = tiles[blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int e = tl.el0 + tid * 4;
  float mx = 0.0f;
  if (e < ld.nq_el) {
    const float* Qp = a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off + e;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int rb = 0; rb < ld.nrb; ++rb) {
      const float4 t = *reinterpret_cast<const float4*>(Qp + (size_t)rb * ld.nq_pad);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    float* dst = a.Qw + (size_t)worker * a.q_stride + ld.q_off + e;
    const int nv = min(4, ld.nq_el - e);
    const float vals[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < nv) {
        dst[i] = vals[i];
        mx = fmaxf(mx, fabsf(vals[i]));
      }
  }
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
    atomicMax(reinterpret_cast<unsigned int*>(a.scaleQ + (size_t)worker * a.L + layer), __float_as_uint(m));
  }
}

// ---------------------------------------------------------------------------
// sweep 2: E_w = M_w - P-bar Q-bar^T (Eq. (7), (8)); worker 0's items also
// write G-hat when the caller asked for it.  Same work items as sweep 1, the
// four wavefronts of a workgroup split the rows.
// ---------------------------------------------------------------------------
template <int RP, int VEC>
__device__ __forceinline__ void residual_tile(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                              float* __restrict__ ghat, int wave, int lane) {
  constexpr int NV = VEC * RP;
  constexpr int U = 8;
  const int cols = ld.cols, r = ld.r;
  const bool exact = (r == RP);
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  const int c = tl.aux * (kWave * VEC) + lane * VEC;
  if (c >= cols) return;
  const int per = (tl.nrows + 3) >> 2;
  const int ra = min(tl.row0 + wave * per, tl.row0 + tl.nrows);
  const int rb = min(ra + per, tl.row0 + tl.nrows);
  float q[NV];
  load_slice<RP, VEC>(a.Qbar + ld.q_off, c, r, exact, q);
  int i = ra;
  for (; i + U <= rb; i += U) {
    Pk<VEC> m[U];
#pragma unroll
    for (int u = 0; u < U; ++u) m[u] = ldv<VEC>(M + (size_t)(i + u) * cols + c);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float p[RP];
      load_row<RP>(Pb, i + u, r, exact, p);
      Pk<VEC> gh, e;
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < RP; ++k) s = fmaf(p[k], q[v * RP + k], s);
        gh.v[v] = s;
        e.v[v] = m[u].v[v] - s;
      }
      stv<VEC>(M + (size_t)(i + u) * cols + c, e);
      if (ghat) stv<VEC>(ghat + (size_t)(i + u) * cols + c, gh);
    }
  }
  for (; i < rb; ++i) {
    const Pk<VEC> m = ldv<VEC>(M + (size_t)i * cols + c);
    float p[RP];
    load_row<RP>(Pb, i, r, exact, p);
    Pk<VEC> gh, e;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      float s = 0.0f;
#pragma unroll
      for (int k = 0; k < RP; ++k) s = fmaf(p[k], q[v * RP + k], s);
      gh.v[v] = s;
      e.v[v] = m.v[v] - s;
    }
    stv<VEC>(M + (size_t)i * cols + c, e);
    if (ghat) stv<VEC>(ghat + (size_t)i * cols + c, gh);
  }
}

template <int RP>
__global__ __launch_bounds__(256) void residual_kernel(DevArgs a, const Tile* __restrict__ tiles, int write_ghat) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  const Tile tl = tiles[blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  float* ghat = nullptr;
  if (write_ghat && worker == 0 && a.ghat) ghat = a.ghat[ld.gidx];
  if (ld.vec == 4)
    residual_tile<RP, 4>(a, ld, tl, worker, ghat, wave, lane);
  else
    residual_tile<RP, 1>(a, ld, tl, worker, ghat, wave, lane);
}

// ---------------------------------------------------------------------------
// 1-D tensors: plain mean over the workers (Eq. (1)).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void vector_mean_kernel(DevArgs a, const VTile* __restrict__ tiles) {
  const VTile tl = tiles[blockIdx.x];
  const VecDesc& vd = a.vecs[tl.vec];
  float* extra = a.ghat ? a.ghat[vd.gidx] : nullptr;
  const float wf = (float)a.W;
  for (int i = 0; i < 4; ++i) {
    const int e = tl.el0 + i * 256 + threadIdx.x;
    if (e < vd.len) {
      float s = 0.0f;
      for (int w = 0; w < a.W; ++w) s += a.grads[(size_t)w * a.n_all + vd.gidx][e];
      s /= wf;
      a.vmean[vd.off + e] = s;
      if (extra) extra[e] = s;
    }
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
#define LQSGD_RP_SWITCH(RPV, CALL)            \
  switch (RPV) {                              \
    case 1: { constexpr int RP = 1; CALL; } break;   \
    case 2: { constexpr int RP = 2; CALL; } break;   \
    case 4: { constexpr int RP = 4; CALL; } break;   \
    case 8: { constexpr int RP = 8; CALL; } break;   \
    case 16: { constexpr int RP = 16; CALL; } break; \
    case 32: { constexpr int RP = 32; CALL; } break; \
    default: return hipErrorInvalidValue;     \
  }

hipError_t launch_add_project(int rp, const DevArgs& a, const Tile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid((ntiles + 3) / 4), block(256);
  LQSGD_RP_SWITCH(rp, (add_project_kernel<RP><<<grid, block, 0, s>>>(a, tiles, ntiles)));
  return hipGetLastError();
}

hipError_t launch_orth(int rp, const DevArgs& a, hipStream_t s) {
  if (a.L <= 0) return hipSuccess;
  const dim3 grid(a.L * a.W), block(256);
  LQSGD_RP_SWITCH(rp, (orth_kernel<RP><<<grid, block, 0, s>>>(a)));
  return hipGetLastError();
}

hipError_t launch_exchange(int mode, int phase, const DevArgs& a, const XTile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid(ntiles), block(256);
  switch (mode) {
    case kQuantOnly: exchange_kernel<kQuantOnly><<<grid, block, 0, s>>>(a, tiles, phase); break;
    case kMeanOnly: exchange_kernel<kMeanOnly><<<grid, block, 0, s>>>(a, tiles, phase); break;
    case kFused: exchange_kernel<kFused><<<grid, block, 0, s>>>(a, tiles, phase); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_back_project(int rp, const DevArgs& a, const Tile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid(ntiles), block(256);
  LQSGD_RP_SWITCH(rp, (back_project_kernel<RP><<<grid, block, 0, s>>>(a, tiles)));
  return hipGetLastError();
}

hipError_t launch_reduce_q(const DevArgs& a, const RTile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  reduce_q_kernel<<<dim3(ntiles), dim3(256), 0, s>>>(a, tiles);
  return hipGetLastError();
}

hipError_t launch_residual(int rp, const DevArgs& a, const Tile* tiles, int ntiles, int write_ghat, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid(ntiles), block(256);
  LQSGD_RP_SWITCH(rp, (residual_kernel<RP><<<grid, block, 0, s>>>(a, tiles, write_ghat)));
  return hipGetLastError();
}

hipError_t launch_vector_mean(const DevArgs& a, const VTile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  vector_mean_kernel<<<dim3(ntiles), dim3(256), 0, s>>>(a, tiles);
  return hipGetLastError();
}

}  // namespace lqsgd
